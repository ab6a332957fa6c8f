// Plain-ALU int4 x int4 GEMM with the dequantising epilogue: one thread per output element.
// Covers every shape (any even d_e, ragged T and N); the fallback for shapes the MFMA kernel
// does not take and the second implementation the tests cross-check it with.
#include "pme_internal.h"

#include <algorithm>

namespace pme {
namespace {

__device__ __forceinline__ int sext4(uint32_t nib) { return ((int)(nib << 28)) >> 28; }

template <bool ASYM>
__global__ void __launch_bounds__(256)
k_gemm_generic(const uint8_t* __restrict__ qx, const uint8_t* __restrict__ qw,
               const float* __restrict__ sx, const float* __restrict__ sw,
               const int32_t* __restrict__ zx, const int32_t* __restrict__ wsum,
               int T, int N, int kb, void* __restrict__ out, int64_t ldo, int out_i32) {
    const int n = blockIdx.x * 16 + (threadIdx.x & 15);
    if (n >= N) return;
    const uint8_t* wr = qw + (int64_t)n * kb;
    // blocks of 16 tokens: the grid's y extent is capped (65535), so a workgroup walks its share of them
    for (int64_t t = (int64_t)blockIdx.y * 16 + (threadIdx.x >> 4); t < T; t += (int64_t)gridDim.y * 16) {
        const uint8_t* ar = qx + t * kb;
        int acc = 0;
        for (int p = 0; p < kb; ++p) {
            const uint32_t av = ar[p], wv = wr[p];
            const int a0 = ASYM ? (int)(av & 0xF) : sext4(av & 0xF);
            const int a1 = ASYM ? (int)(av >> 4) : sext4(av >> 4);
            acc += a0 * sext4(wv & 0xF) + a1 * sext4(wv >> 4);
        }
        if (ASYM) acc -= zx[t] * wsum[n];
        if (out_i32) {
            static_cast<int32_t*>(out)[t * ldo + n] = acc;
        } else {
            const float y = (float)acc * sx[t] * sw[n];
            static_cast<uint16_t*>(out)[t * ldo + n] = f32_to_bf16_bits(y);
        }
    }
}

__global__ void __launch_bounds__(64)
k_weight_rowsum(const uint8_t* __restrict__ qw, int kb, int32_t* __restrict__ wsum) {
    const int n = blockIdx.x, lane = threadIdx.x;
    const uint8_t* wr = qw + (int64_t)n * kb;
    int s = 0;
    for (int p = lane; p < kb; p += 64) {
        const uint32_t wv = wr[p];
        s += sext4(wv & 0xF) + sext4(wv >> 4);
    }
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (lane == 0) wsum[n] = s;
}

// Two 4-bit two's-complement codes per byte, even index in the low nibble.
__global__ void __launch_bounds__(256)
k_pack_int4(const int8_t* __restrict__ codes, int64_t pairs, uint8_t* __restrict__ packed) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < pairs; i += (int64_t)gridDim.x * 256) {
        const uint32_t lo = (uint32_t)codes[2 * i] & 0xFu, hi = (uint32_t)codes[2 * i + 1] & 0xFu;
        packed[i] = (uint8_t)(lo | (hi << 4));
    }
}

}  // namespace

pme_status launch_pack_int4(const int8_t* codes, int64_t pairs, uint8_t* packed, hipStream_t s) {
    const unsigned blocks = (unsigned)std::min<int64_t>((pairs + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(k_pack_int4, dim3(blocks), dim3(256), 0, s, codes, pairs, packed);
    return hip_status(hipGetLastError());
}

pme_status launch_gemm_generic(const GemmArgs& a) {
    if (a.dry) {
        if (a.plan) *a.plan = "k_gemm_generic";
        return PME_OK;
    }
    dim3 grid((unsigned)((a.N + 15) / 16), (unsigned)std::min<int64_t>((a.T + 15) / 16, 65535));
    const int kb = (int)(a.d_e / 2);
    if (a.zx)
        hipLaunchKernelGGL(k_gemm_generic<true>, grid, dim3(256), 0, a.stream, a.qx, a.qw, a.sx, a.sw, a.zx,
                           a.wsum, (int)a.T, (int)a.N, kb, a.y, a.ldy, a.out_i32 ? 1 : 0);
    else
        hipLaunchKernelGGL(k_gemm_generic<false>, grid, dim3(256), 0, a.stream, a.qx, a.qw, a.sx, a.sw, a.zx,
                           a.wsum, (int)a.T, (int)a.N, kb, a.y, a.ldy, a.out_i32 ? 1 : 0);
    return hip_status(hipGetLastError());
}

pme_status launch_weight_rowsum(const uint8_t* qw, int64_t N, int64_t d_e, int32_t* wsum, hipStream_t s) {
    hipLaunchKernelGGL(k_weight_rowsum, dim3((unsigned)N), dim3(64), 0, s, qw, (int)(d_e / 2), wsum);
    return hip_status(hipGetLastError());
}

}  // namespace pme
