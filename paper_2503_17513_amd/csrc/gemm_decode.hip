// W4A4 GEMM for decode shapes (at most 64 tokens, in groups of 16): memory-bound on the packed weights.
//
//   acc[t][n] = sum_j qx[t][j] qw[n][j],  y[t][n] = bf16(acc * sx[t] * sw[n])   (paper Sections 3 and 4).
//
// One workgroup owns 16 output channels and the whole of K; its waves split K into contiguous runs of
// 64-byte chunks (128 codes), so that every weight byte is loaded exactly once, straight from HBM into
// registers, with all of a wave's loads in flight before the first use.  A chunk of 16 channels is one
// global_load_dwordx4 per lane (lane = channel % 16 + 16 * quarter of the chunk) and feeds two
// v_mfma_i32_16x16x64_i8 (even and odd codes, unpacked in registers as in the prefill kernel:
// (w & 0x0F0F0F0F) << 4 and w & 0xF0F0F0F0, accumulator = 256 x the sum).  The tokens are the other MFMA
// operand (rows beyond T repeat the last token and are dropped).  The waves' partial 16 x 16 tiles are
// summed through LDS and the first four waves apply the scales and store bf16.
#include "pme_internal.h"

namespace pme {
namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

enum { MODE_BF16 = 0, MODE_ASYM = 1, MODE_I32 = 2 };

// TG: groups of 16 tokens (T <= 16 TG).  The weight chunks a wave has loaded and unpacked meet the token chunks
// of every group, so the weights are still read exactly once.
// kB: chunks a wave keeps in flight at once (its share of K is ceil(chunks / NW): one round of loads where
// that fits in 8).
template <int NW, int MODE, int TG, int kB>
__global__ void __launch_bounds__(64 * NW)
k_gemm_decode(const uint8_t* __restrict__ qx, const uint8_t* __restrict__ qw,
              const float* __restrict__ sx, const float* __restrict__ sw,
              const int32_t* __restrict__ zx, const int32_t* __restrict__ wsum,
              int T, int N, int kb, void* __restrict__ out, int64_t ldo) {
    __shared__ int part[NW][64][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, kg = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int nchunks = kb >> 6;
    const int c0 = (int)(((int64_t)wave * nchunks) / NW), c1 = (int)(((int64_t)(wave + 1) * nchunks) / NW);
    const uint8_t* wrow = qw + (int64_t)min(n0 + r, N - 1) * kb + kg * 16;
    const uint8_t* xrow[TG];
#pragma unroll
    for (int g = 0; g < TG; ++g) xrow[g] = qx + (int64_t)min(16 * g + r, T - 1) * kb + kg * 16;

    // The epilogue's operands (thread tid < 256 finishes element tid of every group's 16 x 16 tile) are fetched now,
    // together with the weights, so that the epilogue does not start with a dependent round trip to memory.
    const int e_ln = (tid >> 2) & 63, e_i = tid & 3;
    const int e_n = min(n0 + 4 * (e_ln >> 4) + e_i, N - 1);
    float e_sw = 0.f, e_sx[TG] = {};
    int e_ws = 0, e_zx[TG] = {};
    if (tid < 256) {
        if (MODE != MODE_I32) e_sw = sw[e_n];
        if (MODE == MODE_ASYM) e_ws = wsum[e_n];
#pragma unroll
        for (int g = 0; g < TG; ++g) {
            const int t = min(16 * g + (e_ln & 15), T - 1);
            e_sx[g] = MODE != MODE_I32 ? sx[t] : 0.f;
            e_zx[g] = MODE == MODE_ASYM ? zx[t] : 0;
        }
    }

    i32x4 acc[TG];
#pragma unroll
    for (int g = 0; g < TG; ++g) acc[g] = i32x4{0, 0, 0, 0};
    for (int c = c0; c < c1; c += kB) {
        u32x4 w[kB], x[TG][kB];
#pragma unroll
        for (int i = 0; i < kB; ++i) {
            if (c + i < c1) {                           // wave-uniform: surplus slots load nothing
                w[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wrow + (int64_t)(c + i) * 64));
#pragma unroll
                for (int g = 0; g < TG; ++g) x[g][i] = *reinterpret_cast<const u32x4*>(xrow[g] + (int64_t)(c + i) * 64);
            }
        }
#pragma unroll
        for (int i = 0; i < kB; ++i) {
            if (c + i < c1) {
                i32x4 wlo, whi;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    wlo[e] = (int)((w[i][e] & 0x0F0F0F0Fu) << 4);
                    whi[e] = (int)(w[i][e] & 0xF0F0F0F0u);
                }
#pragma unroll
                for (int g = 0; g < TG; ++g) {
                    u32x4 xv = x[g][i];
                    if (MODE == MODE_ASYM) xv ^= 0x88888888u;      // unsigned code u: u ^ 8 as a signed nibble is u - 8
                    i32x4 xlo, xhi;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        xlo[e] = (int)((xv[e] & 0x0F0F0F0Fu) << 4);
                        xhi[e] = (int)(xv[e] & 0xF0F0F0F0u);
                    }
                    acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wlo, xlo, acc[g], 0, 0, 0);
                    acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(whi, xhi, acc[g], 0, 0, 0);
                }
            }
        }
    }
    // one group at a time through the reduction buffer
#pragma unroll
    for (int g = 0; g < TG; ++g) {
        if (g > 0) __syncthreads();                     // the previous group has been read
#pragma unroll
        for (int i = 0; i < 4; ++i) part[wave][lane][i] = acc[g][i];
        __syncthreads();
        if (tid < 256) {
            // element tid = 4 * lane' + i of the 16 x 16 tile: channel 4 * (lane' / 16) + i, token lane' % 16
            const int ln = tid >> 2, i = tid & 3;
            int s = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) s += part[w][ln][i];
            s >>= 8;                                    // exact: the low 8 bits are zero
            const int t = 16 * g + (ln & 15), n = n0 + 4 * (ln >> 4) + i;
            if (t < T && n < N) {
                if (MODE == MODE_ASYM) s -= (e_zx[g] - 8) * e_ws;
                if (MODE == MODE_I32) {
                    static_cast<int32_t*>(out)[(int64_t)t * ldo + n] = s;
                } else {
                    const float y = (float)s * e_sx[g] * e_sw;
                    static_cast<uint16_t*>(out)[(int64_t)t * ldo + n] = f32_to_bf16_bits(y);
                }
            }
        }
    }
}

template <int NW, int TG, int KB>
pme_status launch_kb(const GemmArgs& a) {
    const dim3 grid((unsigned)((a.N + 15) / 16)), block(64 * NW);
    const int kb = (int)(a.d_e / 2);
#define PME_LAUNCH(MODE)                                                                                       \
    hipLaunchKernelGGL((k_gemm_decode<NW, MODE, TG, KB>), grid, block, 0, a.stream, a.qx, a.qw, a.sx, a.sw, a.zx, a.wsum, \
                       (int)a.T, (int)a.N, kb, a.y, a.ldy)
    if (a.out_i32) PME_LAUNCH(MODE_I32);
    else if (a.zx) PME_LAUNCH(MODE_ASYM);
    else PME_LAUNCH(MODE_BF16);
#undef PME_LAUNCH
    return hip_status(hipGetLastError());
}

template <int NW, int TG>
pme_status launch_nw(const GemmArgs& a) {
    // a wave's share of K in one round of loads where registers allow (8 chunks with up to two token groups)
    const int64_t per_wave = (a.d_e / 128 + NW - 1) / NW;
    if constexpr (TG > 2) {
        return launch_kb<NW, TG, 4>(a);
    } else {
        if (per_wave <= 4) return launch_kb<NW, TG, 4>(a);
        if (per_wave <= 6) return launch_kb<NW, TG, 6>(a);
        return launch_kb<NW, TG, 8>(a);
    }
}

template <int TG>
pme_status launch_groups(const GemmArgs& a) {
    const int64_t nchunks = a.d_e / 128;
    if (nchunks >= 32) return launch_nw<16, TG>(a);
    if (nchunks >= 8) return launch_nw<8, TG>(a);
    return launch_nw<4, TG>(a);
}

}  // namespace

pme_status launch_gemm_decode(const GemmArgs& a) {
    // at most 64 tokens, whole 64-byte chunks, 16-byte aligned rows, the x256 accumulator in range
    // (256 * 64 * d_e < 2^31 needs d_e < 2^17; the asymmetric correction is applied after the shift)
    if (a.T > 64 || a.d_e % 128 || a.d_e >= (1 << 17)) return PME_ERR_UNSUPPORTED_PATH;
    if ((reinterpret_cast<uintptr_t>(a.qx) & 15) || (reinterpret_cast<uintptr_t>(a.qw) & 15)) return PME_ERR_UNSUPPORTED_PATH;
    if (a.zx && a.out_i32) return PME_ERR_UNSUPPORTED_PATH;
    if (a.dry) {
        if (a.plan) *a.plan = "k_gemm_decode";
        return PME_OK;
    }
    if (a.T <= 16) return launch_groups<1>(a);
    if (a.T <= 32) return launch_groups<2>(a);
    if (a.T <= 48) return launch_groups<3>(a);
    return launch_groups<4>(a);
}

}  // namespace pme
