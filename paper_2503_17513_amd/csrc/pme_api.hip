// C-ABI entry points: host-side validation and dispatch.  No HIP call is made before the
// arguments have been accepted.
#include "pme_internal.h"

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <mutex>

// Scratch of the entry point that allocates nothing (pme_expanded_linear_static): the quantized activations pass
// through this array instead of a caller's workspace.  Each GPU the library runs on holds its own copy until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[PME_STATIC_SCRATCH_BYTES];

namespace {

std::atomic<int> g_path{PME_PATH_AUTO};

// Device address of `scratch` on the current device, resolved once per device.
constexpr int kMaxScratchDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxScratchDevices] = {};

pme_status scratch_on_current_device(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxScratchDevices) return PME_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return PME_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PME_OK;
}

// Base orders b = q + 1, q a prime power congruent to 3 mod 4 (primes, and 343 = 7^3), with pairwise distinct
// odd parts, so that d_e = b * 2^k has at most one solution.  b = 1: plain power of two.
const int kBaseOrders[] = {1, 12, 20, 60, 68, 72, 132, 140, 152, 312, 344};

bool factor_order(int64_t d_e, int* b, int* k) {
    if (d_e <= 0) return false;
    for (int cand : kBaseOrders) {
        if (d_e % cand) continue;
        int64_t c = d_e / cand;
        if ((c & (c - 1)) != 0) continue;
        int kk = 0;
        while ((int64_t(1) << kk) < c) ++kk;
        *b = cand;
        *k = kk;
        return true;
    }
    return false;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

pme_status check_rotate(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx, int64_t d_e,
                        int* b, int* k) {
    if (xt != PME_F32 && xt != PME_BF16) return PME_ERR_DTYPE;
    if (T < 0 || d <= 0 || d_e <= 0 || d > d_e || ldx < d || (d_e & 1)) return PME_ERR_SHAPE;
    if (T > 0x7FFFFFFF || d_e > (int64_t(1) << 20)) return PME_ERR_SHAPE;
    if (!factor_order(d_e, b, k)) return PME_ERR_UNSUPPORTED_ORDER;
    if (T > 0 && !x) return PME_ERR_NULL;
    if (!aligned(x, xt == PME_F32 ? 4 : 2)) return PME_ERR_ALIGN;
    return PME_OK;
}

pme_status run_rotate(const pme::RotateArgs& a) {
    if (a.T == 0) return PME_OK;
    int path = g_path.load();
    if (path != PME_PATH_GENERIC) {
        pme_status s = pme::launch_rotate_mfma(a);
        if (s != PME_ERR_UNSUPPORTED_PATH || path == PME_PATH_MFMA) return s;
    }
    return pme::launch_rotate_generic(a);
}

pme_status check_gemm(const uint8_t* qx, const uint8_t* qw, int64_t T, int64_t d_e, int64_t N) {
    if (T < 0 || N < 0 || d_e <= 0 || (d_e & 1)) return PME_ERR_SHAPE;
    if (T > 0x7FFFFFFF || N > 0x7FFFFFFF || d_e > (int64_t(1) << 20)) return PME_ERR_SHAPE;
    if (T > 0 && N > 0 && (!qx || !qw)) return PME_ERR_NULL;
    if (!aligned(qx, 4) || !aligned(qw, 4)) return PME_ERR_ALIGN;
    return PME_OK;
}

// Rows of an operand the matrix-core kernels can address with their 32-bit byte offsets, as a multiple of the
// largest tile edge so that a slice starts on a tile (and vector-store) boundary.
int64_t max_slice_rows(int64_t row_bytes) { return std::max<int64_t>(256, (((int64_t(1) << 32) - 1) / row_bytes) & ~int64_t(255)); }

pme_status run_gemm_slice(const pme::GemmArgs& a) {
    int path = g_path.load();
    if (path != PME_PATH_GENERIC) {
        // few tokens: the weight-streaming kernel, unless the output is wide enough to fill the chip with tiles
        const bool stream_weights = a.T <= 16 || (a.T <= 64 && a.N < 8192);       // 64 x 64 tiles: fewer than 128 of them
        pme_status s = stream_weights ? pme::launch_gemm_decode(a) : pme::launch_gemm_mfma(a);
        if (s == PME_ERR_UNSUPPORTED_PATH && stream_weights && a.T > 16) s = pme::launch_gemm_mfma(a);
        if (s != PME_ERR_UNSUPPORTED_PATH || path == PME_PATH_MFMA) return s;
    }
    return pme::launch_gemm_generic(a);
}

// Operands beyond 4 GiB go through the same kernels in slices of tokens (and of output channels).
pme_status run_gemm(const pme::GemmArgs& a) {
    if (a.T == 0 || a.N == 0) return PME_OK;
    const int64_t kb = a.d_e / 2, rows = max_slice_rows(kb), esz = a.out_i32 ? 4 : 2;
    if (a.T <= rows && a.N <= rows) return run_gemm_slice(a);
    for (int64_t t0 = 0; t0 < a.T; t0 += rows)
        for (int64_t n0 = 0; n0 < a.N; n0 += rows) {
            pme::GemmArgs p = a;
            p.T = std::min(rows, a.T - t0);
            p.N = std::min(rows, a.N - n0);
            p.qx = a.qx + t0 * kb;
            p.qw = a.qw + n0 * kb;
            if (a.sx) p.sx = a.sx + t0;
            if (a.sw) p.sw = a.sw + n0;
            if (a.zx) p.zx = a.zx + t0;
            if (a.wsum) p.wsum = a.wsum + n0;
            p.y = static_cast<unsigned char*>(a.y) + (t0 * a.ldy + n0) * esz;
            const pme_status s = run_gemm_slice(p);
            if (s != PME_OK) return s;
        }
    return PME_OK;
}

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

pme_status run_mxgemm_slice(const pme::MxGemmArgs& a) {
    int path = g_path.load();
    if (path != PME_PATH_GENERIC) {
        // few tokens: the weight-streaming kernel, unless the output is wide enough to fill the chip with tiles
        const bool stream_weights = a.T <= 16 || (a.T <= 32 && a.N < 8192);
        pme_status s = stream_weights ? pme::launch_mxgemm_decode(a) : pme::launch_mxgemm_mfma(a);
        if (s == PME_ERR_UNSUPPORTED_PATH && stream_weights) s = pme::launch_mxgemm_mfma(a);
        if (s != PME_ERR_UNSUPPORTED_PATH || path == PME_PATH_MFMA) return s;
    }
    return pme::launch_mxgemm_generic(a);
}

pme_status run_mxgemm(const pme::MxGemmArgs& a) {
    if (a.T == 0 || a.N == 0) return PME_OK;
    const int64_t kb = a.d_e / 2, eb = a.d_e / 32, rows = max_slice_rows(kb);
    if (a.T <= rows && a.N <= rows) return run_mxgemm_slice(a);
    for (int64_t t0 = 0; t0 < a.T; t0 += rows)
        for (int64_t n0 = 0; n0 < a.N; n0 += rows) {
            pme::MxGemmArgs p = a;
            p.T = std::min(rows, a.T - t0);
            p.N = std::min(rows, a.N - n0);
            p.qx = a.qx + t0 * kb;
            p.ex = a.ex + t0 * eb;
            p.qw = a.qw + n0 * kb;
            p.ew = a.ew + n0 * eb;
            p.y = static_cast<unsigned char*>(a.y) + (t0 * a.ldy + n0) * 2;
            const pme_status s = run_mxgemm_slice(p);
            if (s != PME_OK) return s;
        }
    return PME_OK;
}

// Rotate + quantize, then the GEMM on the codes.  Both stages are asked first whether a kernel takes them (a forced
// kernel path may refuse either), so that a refusal launches nothing.
pme_status run_layer(const pme::RotateArgs& ra, const pme::GemmArgs& ga) {
    pme::RotateArgs rd = ra;
    pme::GemmArgs gd = ga;
    rd.dry = gd.dry = true;
    pme_status s = run_rotate(rd);
    if (s != PME_OK) return s;
    if ((s = run_gemm(gd)) != PME_OK) return s;
    if ((s = run_rotate(ra)) != PME_OK) return s;
    return run_gemm(ga);
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

pme_status pme_hadamard_expand_quant(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                     int64_t d_e, uint8_t* qx, float* sx, void* stream) {
    int b, k;
    pme_status s = check_rotate(x, xt, T, d, ldx, d_e, &b, &k);
    if (s != PME_OK) return s;
    if (T > 0 && (!qx || !sx)) return PME_ERR_NULL;
    if (!aligned(qx, 4) || !aligned(sx, 4)) return PME_ERR_ALIGN;
    pme::RotateArgs a{x, xt, T, d, ldx, d_e, b, k, qx, sx, nullptr, nullptr, nullptr, (hipStream_t)stream};
    return run_rotate(a);
}

pme_status pme_expand_quantize_weights(const void* wt, pme_dtype wtype, int64_t N, int64_t d, int64_t ldw,
                                       int64_t d_e, uint8_t* qw, float* sw, void* stream) {
    return pme_hadamard_expand_quant(wt, wtype, N, d, ldw, d_e, qw, sw, stream);
}

pme_status pme_hadamard_expand_quant_asym(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                          int64_t d_e, uint8_t* qx, float* sx, int32_t* zx, void* stream) {
    int b, k;
    pme_status s = check_rotate(x, xt, T, d, ldx, d_e, &b, &k);
    if (s != PME_OK) return s;
    if (T > 0 && (!qx || !sx || !zx)) return PME_ERR_NULL;
    if (!aligned(qx, 4) || !aligned(sx, 4) || !aligned(zx, 4)) return PME_ERR_ALIGN;
    pme::RotateArgs a{x, xt, T, d, ldx, d_e, b, k, qx, sx, zx, nullptr, nullptr, (hipStream_t)stream};
    return run_rotate(a);
}

pme_status pme_hadamard_expand_f32(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                   int64_t d_e, float* xhat, void* stream) {
    int b, k;
    pme_status s = check_rotate(x, xt, T, d, ldx, d_e, &b, &k);
    if (s != PME_OK) return s;
    if (T > 0 && !xhat) return PME_ERR_NULL;
    if (!aligned(xhat, 4)) return PME_ERR_ALIGN;
    pme::RotateArgs a{x, xt, T, d, ldx, d_e, b, k, nullptr, nullptr, nullptr, nullptr, xhat, (hipStream_t)stream};
    return run_rotate(a);
}

pme_status pme_w4a4_gemm(const uint8_t* qx, const float* sx, const uint8_t* qw, const float* sw,
                         int64_t T, int64_t d_e, int64_t N, void* y_bf16, int64_t ldy, void* stream) {
    pme_status s = check_gemm(qx, qw, T, d_e, N);
    if (s != PME_OK) return s;
    if (ldy < N) return PME_ERR_SHAPE;
    if (T > 0 && N > 0 && (!sx || !sw || !y_bf16)) return PME_ERR_NULL;
    if (!aligned(sx, 4) || !aligned(sw, 4) || !aligned(y_bf16, 2)) return PME_ERR_ALIGN;
    pme::GemmArgs a{qx, qw, sx, sw, nullptr, nullptr, T, d_e, N, y_bf16, ldy, false, (hipStream_t)stream};
    return run_gemm(a);
}

pme_status pme_w4a4_gemm_asym(const uint8_t* qx, const float* sx, const int32_t* zx, const uint8_t* qw,
                              const float* sw, const int32_t* wsum, int64_t T, int64_t d_e, int64_t N,
                              void* y_bf16, int64_t ldy, void* stream) {
    pme_status s = check_gemm(qx, qw, T, d_e, N);
    if (s != PME_OK) return s;
    if (ldy < N) return PME_ERR_SHAPE;
    if (T > 0 && N > 0 && (!sx || !sw || !y_bf16 || !zx || !wsum)) return PME_ERR_NULL;
    if (!aligned(sx, 4) || !aligned(sw, 4) || !aligned(y_bf16, 2) || !aligned(zx, 4) || !aligned(wsum, 4))
        return PME_ERR_ALIGN;
    pme::GemmArgs a{qx, qw, sx, sw, zx, wsum, T, d_e, N, y_bf16, ldy, false, (hipStream_t)stream};
    return run_gemm(a);
}

pme_status pme_w4a4_gemm_i32(const uint8_t* qx, const uint8_t* qw, int64_t T, int64_t d_e, int64_t N,
                             int32_t* acc, void* stream) {
    pme_status s = check_gemm(qx, qw, T, d_e, N);
    if (s != PME_OK) return s;
    if (T > 0 && N > 0 && !acc) return PME_ERR_NULL;
    if (!aligned(acc, 4)) return PME_ERR_ALIGN;
    pme::GemmArgs a{qx, qw, nullptr, nullptr, nullptr, nullptr, T, d_e, N, acc, N, true, (hipStream_t)stream};
    return run_gemm(a);
}

pme_status pme_weight_rowsum(const uint8_t* qw, int64_t N, int64_t d_e, int32_t* wsum, void* stream) {
    if (N < 0 || d_e <= 0 || (d_e & 1) || N > 0x7FFFFFFF || d_e > (int64_t(1) << 20)) return PME_ERR_SHAPE;
    if (N > 0 && (!qw || !wsum)) return PME_ERR_NULL;
    if (!aligned(qw, 4) || !aligned(wsum, 4)) return PME_ERR_ALIGN;
    if (N == 0) return PME_OK;
    return pme::launch_weight_rowsum(qw, N, d_e, wsum, (hipStream_t)stream);
}

pme_status pme_pack_int4(const int8_t* codes, int64_t rows, int64_t K, uint8_t* packed, void* stream) {
    if (rows < 0 || K < 0 || (K & 1) || rows > 0x7FFFFFFF || K > (int64_t(1) << 20)) return PME_ERR_SHAPE;
    if (rows > 0 && K > 0 && (!codes || !packed)) return PME_ERR_NULL;
    if (rows == 0 || K == 0) return PME_OK;
    return pme::launch_pack_int4(codes, rows * (K / 2), packed, (hipStream_t)stream);
}

pme_status pme_gemm_plan(int variant, int64_t T, int64_t d_e, int64_t N, char* name, size_t name_len) {
    if (!name || name_len == 0) return PME_ERR_NULL;
    if (variant < 0 || variant > 2) return PME_ERR_DTYPE;
    if (T <= 0 || N <= 0 || d_e <= 0 || (d_e & 1) || (variant == 2 && d_e % 32)) return PME_ERR_SHAPE;
    if (T > 0x7FFFFFFF || N > 0x7FFFFFFF || d_e > (int64_t(1) << 20)) return PME_ERR_SHAPE;
    // operands as the fused calls pass them: 256-byte aligned, never dereferenced by a dry run
    const uint8_t* p8 = reinterpret_cast<const uint8_t*>(uintptr_t(256));
    const float* pf = reinterpret_cast<const float*>(uintptr_t(256));
    const int32_t* pi = reinterpret_cast<const int32_t*>(uintptr_t(256));
    const char* plan = "";
    pme_status s;
    if (variant == 2) {
        pme::MxGemmArgs a{p8, p8, p8, p8, T, d_e, N, const_cast<uint8_t*>(p8), N, nullptr};
        a.dry = true;
        a.plan = &plan;
        s = run_mxgemm(a);
    } else {
        pme::GemmArgs a{p8, p8, pf, pf, variant == 1 ? pi : nullptr, variant == 1 ? pi : nullptr, T, d_e, N,
                        const_cast<uint8_t*>(p8), N, false, nullptr};
        a.dry = true;
        a.plan = &plan;
        s = run_gemm(a);
    }
    if (s != PME_OK) return s;
    snprintf(name, name_len, "%s", plan);
    return PME_OK;
}

size_t pme_workspace_bytes(int64_t T, int64_t d, int64_t d_e, int64_t N) {
    (void)N;
    if (T < 0 || d <= 0 || d_e <= 0 || d > d_e || (d_e & 1)) return 0;
    // packed codes [T, d_e/2], then per-token scales [T] fp32 or MXFP4 scale bytes [T, d_e/32], then the
    // zero points [T] int32 of the asymmetric variant; each 256-byte aligned
    const size_t scales = std::max((size_t)T * sizeof(float), (size_t)T * (size_t)(d_e / 32));
    return round_up((size_t)T * (size_t)(d_e / 2), 256) + round_up(scales, 256) + round_up((size_t)T * sizeof(int32_t), 256);
}

pme_status pme_expanded_linear(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                               int64_t d_e, const uint8_t* qw, const float* sw, int64_t N,
                               void* y_bf16, int64_t ldy, void* workspace, size_t workspace_bytes,
                               void* stream) {
    int b, k;
    pme_status s = check_rotate(x, xt, T, d, ldx, d_e, &b, &k);
    if (s != PME_OK) return s;
    if (N < 0 || N > 0x7FFFFFFF || ldy < N) return PME_ERR_SHAPE;
    if (T > 0 && N > 0 && (!qw || !sw || !y_bf16)) return PME_ERR_NULL;
    if (!aligned(qw, 4) || !aligned(sw, 4) || !aligned(y_bf16, 2)) return PME_ERR_ALIGN;
    size_t need = pme_workspace_bytes(T, d, d_e, N);
    if (T > 0 && !workspace) return PME_ERR_NULL;
    if (!aligned(workspace, 256)) return PME_ERR_ALIGN;
    if (workspace_bytes < need) return PME_ERR_WORKSPACE;
    if (T == 0 || N == 0) return PME_OK;
    uint8_t* qx = static_cast<uint8_t*>(workspace);
    float* sx = reinterpret_cast<float*>(qx + round_up((size_t)T * (size_t)(d_e / 2), 256));
    pme::RotateArgs ra{x, xt, T, d, ldx, d_e, b, k, qx, sx, nullptr, nullptr, nullptr, (hipStream_t)stream};
    pme::GemmArgs ga{qx, qw, sx, sw, nullptr, nullptr, T, d_e, N, y_bf16, ldy, false, (hipStream_t)stream};
    return run_layer(ra, ga);
}

pme_status pme_expanded_linear_static(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                      int64_t d_e, const uint8_t* qw, const float* sw, int64_t N,
                                      void* y_bf16, int64_t ldy, void* stream) {
    int b, k;
    pme_status s = check_rotate(x, xt, T, d, ldx, d_e, &b, &k);
    if (s != PME_OK) return s;
    if (N < 0 || N > 0x7FFFFFFF || ldy < N) return PME_ERR_SHAPE;
    if (T > 0 && N > 0 && (!qw || !sw || !y_bf16)) return PME_ERR_NULL;
    if (!aligned(qw, 4) || !aligned(sw, 4) || !aligned(y_bf16, 2)) return PME_ERR_ALIGN;
    if (pme_workspace_bytes(T, d, d_e, N) > (size_t)PME_STATIC_SCRATCH_BYTES) return PME_ERR_WORKSPACE;
    if (T == 0 || N == 0) return PME_OK;
    void* base = nullptr;
    if ((s = scratch_on_current_device(&base)) != PME_OK) return s;
    // the same layout as the caller's workspace of pme_expanded_linear; the rotation writes every byte the GEMM
    // reads, so nothing left by an earlier call needs clearing
    uint8_t* qx = static_cast<uint8_t*>(base);
    float* sx = reinterpret_cast<float*>(qx + round_up((size_t)T * (size_t)(d_e / 2), 256));
    pme::RotateArgs ra{x, xt, T, d, ldx, d_e, b, k, qx, sx, nullptr, nullptr, nullptr, (hipStream_t)stream};
    pme::GemmArgs ga{qx, qw, sx, sw, nullptr, nullptr, T, d_e, N, y_bf16, ldy, false, (hipStream_t)stream};
    return run_layer(ra, ga);
}

pme_status pme_expanded_linear_asym(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                    int64_t d_e, const uint8_t* qw, const float* sw, const int32_t* wsum,
                                    int64_t N, void* y_bf16, int64_t ldy, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    int b, k;
    pme_status s = check_rotate(x, xt, T, d, ldx, d_e, &b, &k);
    if (s != PME_OK) return s;
    if (N < 0 || N > 0x7FFFFFFF || ldy < N) return PME_ERR_SHAPE;
    if (T > 0 && N > 0 && (!qw || !sw || !wsum || !y_bf16)) return PME_ERR_NULL;
    if (!aligned(qw, 4) || !aligned(sw, 4) || !aligned(wsum, 4) || !aligned(y_bf16, 2)) return PME_ERR_ALIGN;
    const size_t need = pme_workspace_bytes(T, d, d_e, N);
    if (T > 0 && !workspace) return PME_ERR_NULL;
    if (!aligned(workspace, 256)) return PME_ERR_ALIGN;
    if (workspace_bytes < need) return PME_ERR_WORKSPACE;
    if (T == 0 || N == 0) return PME_OK;
    uint8_t* qx = static_cast<uint8_t*>(workspace);
    const size_t scales = std::max((size_t)T * sizeof(float), (size_t)T * (size_t)(d_e / 32));
    float* sx = reinterpret_cast<float*>(qx + round_up((size_t)T * (size_t)(d_e / 2), 256));
    int32_t* zx = reinterpret_cast<int32_t*>(reinterpret_cast<uint8_t*>(sx) + round_up(scales, 256));
    pme::RotateArgs ra{x, xt, T, d, ldx, d_e, b, k, qx, sx, zx, nullptr, nullptr, (hipStream_t)stream};
    pme::GemmArgs ga{qx, qw, sx, sw, zx, wsum, T, d_e, N, y_bf16, ldy, false, (hipStream_t)stream};
    return run_layer(ra, ga);
}

pme_status pme_hadamard_expand_quant_mxfp4(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                           int64_t d_e, uint8_t* qx, uint8_t* ex, void* stream) {
    int b, k;
    pme_status s = check_rotate(x, xt, T, d, ldx, d_e, &b, &k);
    if (s != PME_OK) return s;
    if (d_e % 32) return PME_ERR_SHAPE;
    if (T > 0 && (!qx || !ex)) return PME_ERR_NULL;
    if (!aligned(qx, 4)) return PME_ERR_ALIGN;
    pme::RotateArgs a{x, xt, T, d, ldx, d_e, b, k, qx, nullptr, nullptr, ex, nullptr, (hipStream_t)stream};
    return run_rotate(a);
}

pme_status pme_mxfp4_gemm(const uint8_t* qx, const uint8_t* ex, const uint8_t* qw, const uint8_t* ew,
                          int64_t T, int64_t d_e, int64_t N, void* y_bf16, int64_t ldy, void* stream) {
    if (T < 0 || N < 0 || d_e <= 0 || (d_e % 32) || ldy < N) return PME_ERR_SHAPE;
    if (T > 0x7FFFFFFF || N > 0x7FFFFFFF || d_e > (int64_t(1) << 20)) return PME_ERR_SHAPE;
    if (T > 0 && N > 0 && (!qx || !ex || !qw || !ew || !y_bf16)) return PME_ERR_NULL;
    if (!aligned(qx, 4) || !aligned(qw, 4) || !aligned(y_bf16, 2)) return PME_ERR_ALIGN;
    pme::MxGemmArgs a{qx, ex, qw, ew, T, d_e, N, y_bf16, ldy, (hipStream_t)stream};
    return run_mxgemm(a);
}

pme_status pme_expanded_linear_mxfp4(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                     int64_t d_e, const uint8_t* qw, const uint8_t* ew, int64_t N,
                                     void* y_bf16, int64_t ldy, void* workspace, size_t workspace_bytes,
                                     void* stream) {
    int b, k;
    pme_status s = check_rotate(x, xt, T, d, ldx, d_e, &b, &k);
    if (s != PME_OK) return s;
    if ((d_e % 32) || N < 0 || N > 0x7FFFFFFF || ldy < N) return PME_ERR_SHAPE;
    if (T > 0 && N > 0 && (!qw || !ew || !y_bf16)) return PME_ERR_NULL;
    if (!aligned(qw, 4) || !aligned(y_bf16, 2)) return PME_ERR_ALIGN;
    const size_t need = pme_workspace_bytes(T, d, d_e, N);
    if (T > 0 && !workspace) return PME_ERR_NULL;
    if (!aligned(workspace, 256)) return PME_ERR_ALIGN;
    if (workspace_bytes < need) return PME_ERR_WORKSPACE;
    if (T == 0 || N == 0) return PME_OK;
    uint8_t* qx = static_cast<uint8_t*>(workspace);
    uint8_t* ex = qx + round_up((size_t)T * (size_t)(d_e / 2), 256);
    pme::RotateArgs ra{x, xt, T, d, ldx, d_e, b, k, qx, nullptr, nullptr, ex, nullptr, (hipStream_t)stream};
    pme::MxGemmArgs ga{qx, ex, qw, ew, T, d_e, N, y_bf16, ldy, (hipStream_t)stream};
    // both stages are asked first whether a kernel takes them, so that a refusal launches nothing
    pme::RotateArgs rd = ra;
    pme::MxGemmArgs gd = ga;
    rd.dry = gd.dry = true;
    if ((s = run_rotate(rd)) != PME_OK || (s = run_mxgemm(gd)) != PME_OK) return s;
    s = run_rotate(ra);
    if (s != PME_OK) return s;
    return run_mxgemm(ga);
}

pme_status pme_factor_order(int64_t d_e, int32_t* b, int32_t* k) {
    if (!b || !k) return PME_ERR_NULL;
    int bb, kk;
    if (!factor_order(d_e, &bb, &kk)) return PME_ERR_UNSUPPORTED_ORDER;
    *b = bb;
    *k = kk;
    return PME_OK;
}

pme_status pme_base_block(int64_t b, int8_t* out) {
    if (!out) return PME_ERR_NULL;
    bool known = false;
    for (int cand : kBaseOrders) known = known || (cand == b);
    if (!known) return PME_ERR_UNSUPPORTED_ORDER;
    if (b == 1) { out[0] = 1; return PME_OK; }
    const int q = (int)b - 1;
    // quadratic character of GF(q) by marking the squares
    int8_t chi[512];
    for (int i = 0; i < q; ++i) chi[i] = -1;
    chi[0] = 0;
    for (int i = 1; i < q; ++i) chi[pme::gf_square(q, i)] = 1;
    for (int a = 0; a < b; ++a)
        for (int ap = 0; ap < b; ++ap) {
            int v;
            if (a == 0) v = 1;
            else if (ap == 0) v = -1;
            else if (a == ap) v = 1;
            else v = chi[pme::gf_sub(q, a - 1, ap - 1)];
            out[a * b + ap] = (int8_t)v;
        }
    return PME_OK;
}

pme_status pme_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst) return PME_ERR_NULL;
    if (bytes % 16) return PME_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(dst, 16)) return PME_ERR_ALIGN;
    if (bytes == 0) return PME_OK;
    return pme::launch_probe_copy(src, dst, bytes, (hipStream_t)stream);
}

pme_status pme_probe_read(const void* src, size_t bytes, uint32_t* sink, size_t sink_elems, void* stream) {
    if (!src || !sink) return PME_ERR_NULL;
    if (bytes % 16 || sink_elems < (size_t)pme::kProbeStreamBlocks * 256) return PME_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(sink, 4)) return PME_ERR_ALIGN;
    return pme::launch_probe_read(src, bytes, sink, (hipStream_t)stream);
}

pme_status pme_probe_launch(void* stream) { return pme::launch_probe_empty((hipStream_t)stream); }

pme_status pme_probe_mfma(int kind, int32_t* out, size_t out_elems, int iters, double* ops, void* stream) {
    if (!out) return PME_ERR_NULL;
    if (kind < 0 || kind > 3) return PME_ERR_DTYPE;
    if (iters < 0 || iters > (1 << 24) || out_elems < (size_t)pme::kProbeMfmaBlocks * 256) return PME_ERR_SHAPE;
    if (!aligned(out, 4)) return PME_ERR_ALIGN;
    if (kind >= 2) iters = (iters + 3) / 4 * 4;           // the random-code loops run in rounds of four iterations
    if (ops) *ops = (double)pme::kProbeMfmaBlocks * 4 * 4 * (double)iters * ((kind & 1) == 0 ? 65536.0 : 131072.0);
    return pme::launch_probe_mfma(kind, out, iters, (hipStream_t)stream);
}

void pme_set_gemm_tile(int id) {
    if (id >= 100) { pme::set_mxgemm_tile_override(id - 100); return; }
    pme::set_gemm_tile_override(id);
    if (id == 0) pme::set_mxgemm_tile_override(0);
}
void pme_set_path(pme_path p) { g_path.store((int)p); }
pme_path pme_get_path(void) { return (pme_path)g_path.load(); }

const char* pme_status_string(pme_status s) {
    switch (s) {
        case PME_OK: return "ok";
        case PME_ERR_NULL: return "null pointer";
        case PME_ERR_SHAPE: return "bad shape";
        case PME_ERR_UNSUPPORTED_ORDER: return "unsupported Hadamard order";
        case PME_ERR_ALIGN: return "misaligned pointer or pitch";
        case PME_ERR_WORKSPACE: return "workspace too small";
        case PME_ERR_DTYPE: return "unknown dtype";
        case PME_ERR_HIP: return "HIP launch failed";
        case PME_ERR_UNSUPPORTED_PATH: return "no kernel path (or not the forced one) covers this shape";
        case PME_ERR_COLD_SHAPE: return "first use of this shape cannot happen under stream capture";
    }
    return "unknown status";
}

int pme_version(void) { return 100; }

#pragma GCC visibility pop
}  // extern "C"
