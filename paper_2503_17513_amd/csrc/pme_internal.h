// Internal declarations shared by the translation units of libpme (not installed).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>
#include <utility>
#include <stdint.h>
#include "../../include/pme.h"

namespace pme {

struct RotateArgs {
    const void* x;
    pme_dtype xt;
    int64_t T, d, ldx, d_e;
    int b, k;            // d_e = b * 2^k
    uint8_t* qx;         // packed codes out (may be null when only xhat is wanted)
    float* sx;           // scales out
    int32_t* zx;         // zero points out (asymmetric quantizer) or null
    uint8_t* ex;         // MXFP4: E8M0 scale bytes out [T, d_e / 32] (then qx holds E2M1 codes, sx is unused)
    float* xhat;         // fp32 rotated activations out (debug) or null
    hipStream_t stream;
    int fold = 0;        // set by the MFMA launcher: butterfly stages folded into the base block (then b, k describe the folded shape)
    bool dry = false;    // only answer whether a kernel takes the shape: nothing is launched, no table is built
};

struct MxGemmArgs {
    const uint8_t* qx;   // [T, d_e / 2] packed E2M1
    const uint8_t* ex;   // [T, d_e / 32] E8M0
    const uint8_t* qw;   // [N, d_e / 2]
    const uint8_t* ew;   // [N, d_e / 32]
    int64_t T, d_e, N;
    void* y;             // bf16 [T, ldy]
    int64_t ldy;
    hipStream_t stream;
    bool dry = false;    // only answer whether a kernel takes the shape: nothing is launched
    const char** plan = nullptr;   // dry runs: receives the name of the kernel configuration that would run
};
pme_status launch_mxgemm_generic(const MxGemmArgs& a);
pme_status launch_mxgemm_mfma(const MxGemmArgs& a);
pme_status launch_mxgemm_decode(const MxGemmArgs& a);

struct GemmArgs {
    const uint8_t* qx;
    const uint8_t* qw;
    const float* sx;     // null for the int32 debug output
    const float* sw;
    const int32_t* zx;   // asymmetric: zero points and weight row sums, else null
    const int32_t* wsum;
    int64_t T, d_e, N;
    void* y;             // bf16 [T, ldy] or int32 [T, N]
    int64_t ldy;
    bool out_i32;
    hipStream_t stream;
    bool dry = false;    // only answer whether a kernel takes the shape: nothing is launched
    const char** plan = nullptr;   // dry runs: receives the name of the kernel configuration that would run
};

// Each launcher returns PME_ERR_UNSUPPORTED_PATH when the shape is outside what its kernels cover.
pme_status launch_rotate_generic(const RotateArgs& a);
pme_status launch_rotate_mfma(const RotateArgs& a);
pme_status launch_gemm_generic(const GemmArgs& a);
pme_status launch_gemm_mfma(const GemmArgs& a);
pme_status launch_gemm_decode(const GemmArgs& a);
pme_status launch_weight_rowsum(const uint8_t* qw, int64_t N, int64_t d_e, int32_t* wsum, hipStream_t s);
pme_status launch_pack_int4(const int8_t* codes, int64_t pairs, uint8_t* packed, hipStream_t s);
pme_status launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s);
constexpr int kProbeStreamBlocks = 256 * 8;   // workgroups of 256 threads the streaming probes launch (8 per compute unit)
pme_status launch_probe_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s);
pme_status launch_probe_empty(hipStream_t s);
constexpr int kProbeMfmaBlocks = 512;   // workgroups of 256 threads the matrix-core probe launches
pme_status launch_probe_mfma(int kind, int32_t* out, int iters, hipStream_t s);
void set_gemm_tile_override(int id);
void set_rotate_tpw_override(int tpw);
void set_mxgemm_tile_override(int id);

// Lets `kern` be launched with up to `bytes` of dynamic LDS.  The attribute is set once per kernel and
// device (`done` holds one bit per device and belongs to the kernel's launcher), not on every launch.
template <class K> inline pme_status allow_dynamic_lds(K kern, int bytes, std::atomic<uint32_t>& done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PME_ERR_HIP;
    const uint32_t bit = 1u << (dev & 31);
    if (done.load(std::memory_order_acquire) & bit) return PME_OK;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        return PME_ERR_HIP;
    done.fetch_or(bit, std::memory_order_release);
    return PME_OK;
}

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}).
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

inline pme_status hip_status(hipError_t e) { return e == hipSuccess ? PME_OK : PME_ERR_HIP; }

// Workgroup -> output tile map of the tiled GEMMs.  Workgroups are dealt round-robin to the 8 XCDs, each with
// an L2 of its own, so XCD x (= workgroup index % 8) gets a compact sub-grid of tiles: the XCDs form a
// gm x (8 / gm) grid over the tile grid and XCD x walks its tiles_m / gm by tiles_n / (8 / gm) part row by row.
// What one L2 must fetch is then (rows of qx + rows of qw) of that part rather than of whole tile rows.
// xcd_grid_m picks gm (the split with the fewest operand rows per XCD); 0 = no split fits, identity map.
inline int xcd_grid_m(int tiles_m, int tiles_n, int bm, int bn) {
    int best = 0;
    long best_rows = 0;
    for (int gm = 1; gm <= 8; gm *= 2) {
        const int gn = 8 / gm;
        if (tiles_m % gm || tiles_n % gn) continue;
        const long rows = (long)(tiles_m / gm) * bm + (long)(tiles_n / gn) * bn;
        if (!best || rows < best_rows) { best = gm; best_rows = rows; }
    }
    return best;
}
__device__ __forceinline__ void xcd_tile(int wg, int tiles_m, int tiles_n, int gm, int& tm, int& tn) {
    if (gm == 0) { tm = wg / tiles_n; tn = wg % tiles_n; return; }
    const int gn = 8 / gm, pn = tiles_n / gn, pm = tiles_m / gm;
    const int x = wg & 7, i = wg >> 3;
    tm = (x / gn) * pm + i / pn;
    tn = (x % gn) * pn + i % pn;
}

// Round-to-nearest-even float -> bf16 bits (finite inputs; NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// E8M0 byte and power-of-two scale of an MXFP4 block whose largest magnitude is amax (>= 0, finite):
// shared exponent floor(log2 amax) - 2 (2 = largest exponent of E2M1), byte = exponent + 127 clamped at 0.
__device__ __forceinline__ uint32_t mx_scale_byte(float amax) {
    const int e = (int)((__float_as_uint(amax) >> 23) & 0xFFu);   // biased exponent; 0 for zero / subnormal
    return (uint32_t)max(e - 2, 0);
}
__device__ __forceinline__ float mx_scale_value(uint32_t byte) {
    return __uint_as_float(byte ? (byte << 23) : 0x00400000u);    // 2^(byte - 127)
}

// Eight values divided by the power-of-two scale X and converted to E2M1 (round half to even, saturating),
// packed in one dword, first value in the lowest nibble.
__device__ __forceinline__ uint32_t mx_pack8(float f0, float f1, float f2, float f3, float f4, float f5, float f6,
                                             float f7, float X) {
    uint32_t w = 0;
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, f0, f1, X, 0);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, f2, f3, X, 1);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, f4, f5, X, 2);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, f6, f7, X, 3);
    return w;
}

// Entry P[a][ap] of the Paley type-I block I + [[0, 1^T], [-1, Q]], Q[i][j] = chi((i - j) mod q),
// given the table chi[0..q-1] of the quadratic character.  b = q + 1.
// Field arithmetic behind the Paley blocks, by element number: GF(q) for the primes q = b - 1 in use (the
// residues) and GF(343) = GF(7)[t] / (t^3 + t + 1), where c0 + 7 c1 + 49 c2 stands for c0 + c1 t + c2 t^2
// (the cubic has no root in GF(7), hence is irreducible).
__host__ __device__ inline int gf_sub(int q, int i, int j) {
    if (q != 343) {
        const int d = i - j;
        return d < 0 ? d + q : d;
    }
    const int d0 = (i % 7 - j % 7 + 7) % 7, d1 = ((i / 7) % 7 - (j / 7) % 7 + 7) % 7, d2 = (i / 49 - j / 49 + 7) % 7;
    return d0 + 7 * d1 + 49 * d2;
}
__host__ __device__ inline int gf_square(int q, int i) {
    if (q != 343) return (int)(((long long)i * i) % q);
    const int a0 = i % 7, a1 = (i / 7) % 7, a2 = i / 49;
    // (a0 + a1 t + a2 t^2)^2, then t^4 = -t^2 - t and t^3 = -t - 1
    int p0 = a0 * a0, p1 = 2 * a0 * a1, p2 = 2 * a0 * a2 + a1 * a1, p3 = 2 * a1 * a2, p4 = a2 * a2;
    p2 -= p4; p1 -= p4;
    p1 -= p3; p0 -= p3;
    p0 = ((p0 % 7) + 7) % 7; p1 = ((p1 % 7) + 7) % 7; p2 = ((p2 % 7) + 7) % 7;
    return p0 + 7 * p1 + 49 * p2;
}
// Quadratic character table of GF(q): chi[0] = 0, +1 at the non-zero squares, -1 elsewhere.  Called by every
// thread of a workgroup (thread tid of nthreads); the table is complete when the call returns.
__device__ inline void fill_quadratic_character(signed char* chi, int q, int tid, int nthreads) {
    for (int i = tid; i < q; i += nthreads) chi[i] = (i == 0) ? 0 : -1;
    __syncthreads();
    for (int i = 1 + tid; i < q; i += nthreads) chi[gf_square(q, i)] = 1;
    __syncthreads();
}

// Entry (a, a') of the Paley block P = I + [[0, 1^T], [-1, Q]], Q[i][j] = chi(x_i - x_j), block index a >= 1
// standing for field element a - 1.
__device__ __forceinline__ int paley_entry(const signed char* chi, int q, int a, int ap) {
    if (a == 0) return 1;
    if (ap == 0) return -1;
    if (a == ap) return 1;
    return chi[gf_sub(q, a - 1, ap - 1)];
}

}  // namespace pme
