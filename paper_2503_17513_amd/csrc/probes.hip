// Measurement probes: kernels of known size that give the measured ceilings the hot-path kernels are
// priced against next to the published ones, and calibrate the profiler's byte counters.
//   k_probe_copy  plain streaming copy (HBM read + write), four 16-byte loads in flight per lane.
//   k_probe_read  read-only stream of the same shape (the rotate + quantize stage is four fifths reads).
//   k_probe_empty a kernel that does nothing: the cost of a dependent launch, the floor of a chain of tiny kernels.
//   k_probe_mfma  back-to-back independent matrix-core instructions with nothing else in the loop:
//                 the rate the matrix pipe sustains at the clock the chip actually holds under that load.
//                 That rate depends on the operands' bit activity (the pipe is power-limited), so the probe runs
//                 on near-constant operands (which reach the published peak) and on pseudo-random codes.
#include "pme_internal.h"

namespace pme {
namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Each workgroup walks 16 KB pieces (4 x 16 bytes per lane, all four loads issued before the first store); the
// chunks beyond the last whole piece are copied one per lane.
__global__ void __launch_bounds__(256)
k_probe_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
    const size_t whole = n16 / 1024 * 1024;
    for (size_t p = (size_t)blockIdx.x * 1024; p < whole; p += (size_t)gridDim.x * 1024) {
        const size_t i = p + threadIdx.x;
        const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + 256);
        const u32x4 c = __builtin_nontemporal_load(src + i + 512), d = __builtin_nontemporal_load(src + i + 768);
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + 256);
        __builtin_nontemporal_store(c, dst + i + 512);
        __builtin_nontemporal_store(d, dst + i + 768);
    }
    for (size_t i = whole + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ void __launch_bounds__(256)
k_probe_read(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
    const size_t whole = n16 / 1024 * 1024;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t p = (size_t)blockIdx.x * 1024; p < whole; p += (size_t)gridDim.x * 1024) {
        const size_t i = p + threadIdx.x;
        const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + 256);
        const u32x4 c = __builtin_nontemporal_load(src + i + 512), d = __builtin_nontemporal_load(src + i + 768);
        acc.x ^= a.x ^ b.x ^ c.x ^ d.x;
        acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
        acc.z ^= a.z ^ b.z ^ c.z ^ d.z;
        acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
    }
    for (size_t i = whole + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) acc.x ^= src[i].x ^ src[i].y ^ src[i].z ^ src[i].w;
    // the result depends on every load; each lane stores it (the probe's only writes: 4 bytes per lane)
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

__global__ void k_probe_empty() {}

__device__ __forceinline__ uint32_t probe_rand(uint32_t& state) {
    state = state * 1664525u + 1013904223u;         // a linear congruential step; the high half is the usable part
    return state;
}

// Four independent accumulator chains per wave, so that the pipe never waits on a result.
// KIND 0: v_mfma_i32_32x32x32_i8 (65536 ops each).  KIND 1: v_mfma_scale_f32_32x32x64_f8f6f4 with FP4
// operands (131072 flops each).  The operands are small integers / small E2M1 codes; sums stay finite.
// KIND 2 / 3: the same two instructions on pseudo-random codes -- for int8 the bytes the int4 GEMM feeds the
// pipe (a random nibble times 16), for FP4 random E2M1 codes -- over four operand register sets that rotate
// against the accumulators, so that consecutive instructions toggle the operand buses as a GEMM does.
template <int KIND>
__global__ void __launch_bounds__(256) k_probe_mfma(int32_t* __restrict__ out, int iters) {
    const int t = (int)threadIdx.x;
    int32_t s = 0;
    if constexpr (KIND == 2 || KIND == 3) {
        uint32_t state = 12345u + (uint32_t)t * 7919u + blockIdx.x * 104729u;
        i32x8 a[4], b[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint32_t ra = (probe_rand(state) >> 16) | (probe_rand(state) & 0xFFFF0000u);
                uint32_t rb = (probe_rand(state) >> 16) | (probe_rand(state) & 0xFFFF0000u);
                if (KIND == 2) { ra &= 0xF0F0F0F0u; rb &= 0xF0F0F0F0u; }
                a[q][e] = e < 4 ? (int)ra : 0;
                b[q][e] = e < 4 ? (int)rb : 0;
            }
        if constexpr (KIND == 2) {
            i32x16 c[4] = {{0}, {0}, {0}, {0}};
            // rounds of 16 instructions with compile-time register numbers (iters is rounded up to a multiple of 4)
            for (int it = 0; it < iters; it += 4) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const i32x8& ar = a[(q + r) & 3];
                        const i32x4 aq = {ar[0], ar[1], ar[2], ar[3]};
                        const i32x4 bq = {b[q][0], b[q][1], b[q][2], b[q][3]};
                        c[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aq, bq, c[q], 0, 0, 0);
                    }
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) s += c[0][e] + c[1][e] + c[2][e] + c[3][e];
        } else {
            f32x16 c[4] = {{0}, {0}, {0}, {0}};
            for (int it = 0; it < iters; it += 4) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        c[q] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[(q + r) & 3], b[q], c[q], 4, 4, 0, 120, 0, 120);
            }
            float f = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) f += c[0][e] + c[1][e] + c[2][e] + c[3][e];
            s = (int32_t)__float_as_uint(f);
        }
    } else if constexpr (KIND == 0) {
        const i32x4 a = {0x01010101 * (t & 3), 0x01000100, 0x00010001, 0x01010101};
        const i32x4 b = {0x01010101, 0x00010001, 0x01000100, 0x01010101 * ((t >> 2) & 1)};
        i32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
        for (int it = 0; it < iters; ++it) {
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) s += c0[e] + c1[e] + c2[e] + c3[e];
    } else {
        // E2M1 codes 0x2 = 1.0, 0x1 = 0.5, 0x0 = 0; scale byte 120 = 2^-7 keeps the sums small
        const i32x8 a = {0x22222222, 0x11111111 * (t & 1), 0x20202020, 0x02020202, 0, 0, 0, 0};
        const i32x8 b = {0x12121212, 0x22222222, 0x11111111 * ((t >> 1) & 1), 0x21212121, 0, 0, 0, 0};
        f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
        for (int it = 0; it < iters; ++it) {
            c0 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c0, 4, 4, 0, 120, 0, 120);
            c1 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c1, 4, 4, 0, 120, 0, 120);
            c2 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c2, 4, 4, 0, 120, 0, 120);
            c3 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c3, 4, 4, 0, 120, 0, 120);
        }
        float f = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) f += c0[e] + c1[e] + c2[e] + c3[e];
        s = (int32_t)__float_as_uint(f);
    }
    out[(size_t)blockIdx.x * 256 + t] = s;
}

}  // namespace

pme_status launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 1023) / 1024;
    if (blocks > (size_t)kProbeStreamBlocks) blocks = kProbeStreamBlocks;
    hipLaunchKernelGGL(k_probe_copy, dim3((unsigned)blocks), dim3(256), 0, s, (const u32x4*)src, (u32x4*)dst, n16);
    return hip_status(hipGetLastError());
}

pme_status launch_probe_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s) {
    hipLaunchKernelGGL(k_probe_read, dim3(kProbeStreamBlocks), dim3(256), 0, s, (const u32x4*)src, bytes / 16, sink);
    return hip_status(hipGetLastError());
}

pme_status launch_probe_empty(hipStream_t s) {
    hipLaunchKernelGGL(k_probe_empty, dim3(1), dim3(64), 0, s);
    return hip_status(hipGetLastError());
}

pme_status launch_probe_mfma(int kind, int32_t* out, int iters, hipStream_t s) {
    // 512 workgroups of 4 waves: two waves on every SIMD of the 256 compute units
    if (kind == 0) hipLaunchKernelGGL(k_probe_mfma<0>, dim3(kProbeMfmaBlocks), dim3(256), 0, s, out, iters);
    else if (kind == 1) hipLaunchKernelGGL(k_probe_mfma<1>, dim3(kProbeMfmaBlocks), dim3(256), 0, s, out, iters);
    else if (kind == 2) hipLaunchKernelGGL(k_probe_mfma<2>, dim3(kProbeMfmaBlocks), dim3(256), 0, s, out, iters);
    else hipLaunchKernelGGL(k_probe_mfma<3>, dim3(kProbeMfmaBlocks), dim3(256), 0, s, out, iters);
    return hip_status(hipGetLastError());
}

}  // namespace pme
