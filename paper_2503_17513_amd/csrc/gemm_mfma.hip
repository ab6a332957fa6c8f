// W4A4 GEMM on the int8 matrix cores with the dequantising epilogue fused in.
//
//   acc[t][n] = sum_j qx[t][j] qw[n][j]   (paper Section 3: Q(X_hat) Q(W_hat)),
//   y[t][n]   = bf16(acc * sx[t] * sw[n]) (Section 4: per-token and per-channel scales).
//
// Both operands are K-contiguous packed int4.  A workgroup owns a BM x BN output tile and walks
// K in steps of 128 codes (64 packed bytes per row).  Packed bytes go HBM -> registers -> LDS
// (double buffered); a wave reads 16 packed bytes per lane (32 codes) with one ds_read_b128 and
// unpacks them in registers into two int8 MFMA operands:
//     even codes:  (w & 0x0F0F0F0F) << 4      odd codes:  w & 0xF0F0F0F0
// A nibble moved to the top of a byte is 16 x its two's-complement value, so no sign extension
// is needed; both operands carry the factor 16 and the int32 accumulator holds 256 x the exact
// sum (|256 acc| <= 256 * 64 * d_e < 2^31 for d_e <= 2^17), removed in the epilogue.
// The order in which codes meet inside an MFMA is the same permutation for both operands, which
// an exact integer sum does not notice.
#include "pme_internal.h"

namespace pme {
namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kRowBytes = 64;     // packed bytes per tile row per K step (128 codes)
constexpr int kThreads = 256;

// LDS swizzle: the 16-byte chunk kc (0..3) of tile row r is stored at chunk kc ^ swz(r), so that
// the 16 or 32 rows read together by a ds_read_b128 spread over all banks.
__device__ __forceinline__ int swz(int r) { return ((r >> 1) ^ (r >> 3)) & 3; }

template <int BM, int BN, int WM, int WN, bool OUT_I32, bool ASYM>
__global__ void __launch_bounds__(kThreads)
k_gemm_mfma(const uint8_t* __restrict__ qx, const uint8_t* __restrict__ qw,
            const float* __restrict__ sx, const float* __restrict__ sw,
            const int32_t* __restrict__ zx, const int32_t* __restrict__ wsum,
            int T, int N, int kb, void* __restrict__ out, int64_t ldo, int tiles_m, int tiles_n) {
    static_assert((BM / WM) * (BN / WN) == kThreads / 64, "four waves");
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int ROWS = BM + BN;
    constexpr int CHUNKS = ROWS * 4 / kThreads;     // 16-byte chunks each thread moves per K step
    static_assert(ROWS * 4 % kThreads == 0, "tile rows");
    constexpr int STAGE = ROWS * kRowBytes;

    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / (BN / WN), wn = wave % (BN / WN);

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tiles so
    // that tiles sharing rows of qx / qw share an L2.
    int tile = blockIdx.x;
    const int ntiles = tiles_m * tiles_n;
    if ((ntiles & 7) == 0) tile = (blockIdx.x & 7) * (ntiles >> 3) + (blockIdx.x >> 3);
    const int tm = tile / tiles_n, tn = tile % tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;

    // global source of each chunk this thread moves
    const uint8_t* src[CHUNKS];
    int dst_off[CHUNKS];
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const int cid = tid + kThreads * i;
        const int r = cid >> 2, kc = cid & 3;
        const uint8_t* base;
        if (r < BM) base = qx + (int64_t)min(m0 + r, T - 1) * kb;
        else base = qw + (int64_t)min(n0 + r - BM, N - 1) * kb;
        src[i] = base + kc * 16;
        dst_off[i] = r * kRowBytes + ((kc ^ swz(r)) << 4);
    }

    i32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    const int KT = kb / kRowBytes;
    u32x4 stage_regs[CHUNKS];
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) stage_regs[i] = *reinterpret_cast<const u32x4*>(src[i]);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) *reinterpret_cast<u32x4*>(smem + dst_off[i]) = stage_regs[i];
    __syncthreads();

    const int frow = lane & 31, fk = lane >> 5;
    for (int kt = 0; kt < KT; ++kt) {
        const unsigned char* cur = smem + (kt & 1) * STAGE;
        if (kt + 1 < KT) {
#pragma unroll
            for (int i = 0; i < CHUNKS; ++i)
                stage_regs[i] = *reinterpret_cast<const u32x4*>(src[i] + (int64_t)(kt + 1) * kRowBytes);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            i32x4 alo[FM], ahi[FM], blo[FN], bhi[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const int r = wm * WM + 32 * i + frow;
                u32x4 w = *reinterpret_cast<const u32x4*>(cur + r * kRowBytes + (((2 * s + fk) ^ swz(r)) << 4));
                // unsigned codes u: u ^ 8 read as a signed nibble is u - 8; the epilogue adds 8 * wsum back
                if (ASYM) w ^= 0x88888888u;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    alo[i][e] = (int)((w[e] & 0x0F0F0F0Fu) << 4);
                    ahi[i][e] = (int)(w[e] & 0xF0F0F0F0u);
                }
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int r = BM + wn * WN + 32 * j + frow;
                const u32x4 w = *reinterpret_cast<const u32x4*>(cur + r * kRowBytes + (((2 * s + fk) ^ swz(r)) << 4));
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    blo[j][e] = (int)((w[e] & 0x0F0F0F0Fu) << 4);
                    bhi[j][e] = (int)(w[e] & 0xF0F0F0F0u);
                }
            }
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], blo[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bhi[j], acc[i][j], 0, 0, 0);
                }
        }
        if (kt + 1 < KT) {
            unsigned char* nxt = smem + ((kt + 1) & 1) * STAGE;
#pragma unroll
            for (int i = 0; i < CHUNKS; ++i) *reinterpret_cast<u32x4*>(nxt + dst_off[i]) = stage_regs[i];
        }
        __syncthreads();
    }

    // Epilogue.  Accumulator element e of a 32x32 block: row 8 (e / 4) + 4 (lane / 32) + e % 4, column lane % 32.
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = n0 + wn * WN + 32 * j + frow;
        if (n >= N) continue;
        float swn = 0.f;
        int ws = 0;
        if (!OUT_I32) swn = sw[n];
        if (ASYM) ws = wsum[n];
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = m0 + wm * WM + 32 * i + 8 * (e >> 2) + 4 * fk + (e & 3);
                if (t >= T) continue;
                int a = acc[i][j][e] >> 8;      // exact: the low 8 bits are zero
                if (ASYM) a -= (zx[t] - 8) * ws;
                if (OUT_I32) {
                    static_cast<int32_t*>(out)[(int64_t)t * ldo + n] = a;
                } else {
                    const float y = (float)a * sx[t] * swn;
                    static_cast<uint16_t*>(out)[(int64_t)t * ldo + n] = f32_to_bf16_bits(y);
                }
            }
        }
    }
}

template <int BM, int BN, int WM, int WN>
pme_status launch_tile(const GemmArgs& a) {
    const int tiles_m = (int)((a.T + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const int kb = (int)(a.d_e / 2);
    const size_t lds = 2 * (size_t)(BM + BN) * kRowBytes;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(kThreads);
#define PME_LAUNCH(I32, AS)                                                                              \
    hipLaunchKernelGGL((k_gemm_mfma<BM, BN, WM, WN, I32, AS>), grid, block, lds, a.stream, a.qx, a.qw, a.sx, \
                       a.sw, a.zx, a.wsum, (int)a.T, (int)a.N, kb, a.y, a.ldy, tiles_m, tiles_n)
    if (a.out_i32) PME_LAUNCH(true, false);
    else if (a.zx) PME_LAUNCH(false, true);
    else PME_LAUNCH(false, false);
#undef PME_LAUNCH
    return hip_status(hipGetLastError());
}

}  // namespace

pme_status launch_gemm_mfma(const GemmArgs& a) {
    // d_e a multiple of 128 (whole K steps), 16-byte aligned rows, and the x256 accumulator in range.
    if (a.d_e % 128 || a.d_e > (1 << 17)) return PME_ERR_UNSUPPORTED_PATH;
    if ((reinterpret_cast<uintptr_t>(a.qx) & 15) || (reinterpret_cast<uintptr_t>(a.qw) & 15)) return PME_ERR_UNSUPPORTED_PATH;
    if (a.zx && a.out_i32) return PME_ERR_UNSUPPORTED_PATH;
    // Tile choice: the largest tile that still gives every one of the 256 compute units a workgroup.
    const int64_t cus = 256;
    auto tiles = [&](int bm, int bn) { return ((a.T + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
    if (tiles(256, 256) >= cus) return launch_tile<256, 256, 128, 128>(a);
    if (tiles(128, 256) >= cus) return launch_tile<128, 256, 64, 128>(a);
    if (tiles(128, 192) >= cus) return launch_tile<128, 192, 64, 96>(a);
    if (tiles(128, 128) >= cus) return launch_tile<128, 128, 64, 64>(a);
    if (tiles(64, 128) >= cus / 2) return launch_tile<64, 128, 32, 64>(a);
    return launch_tile<64, 64, 32, 32>(a);
}

}  // namespace pme
