// Plain-ALU rotate + quantize kernel: one workgroup per token, every supported shape.
// It is the fallback for shapes the MFMA kernel does not cover (2^k < 32, odd d, 2^k > 512)
// and an independent second implementation that the tests cross-check the MFMA kernel with.
//
// Per token (paper Section 3, X_hat = X H_hat with H = P_b (x) S_{2^k}):
//   Z[a'][c] = sum_a P[a][a'] x[a 2^k + c]        (base block, only rows a with a 2^k + c < d)
//   U[a'][:] = FWHT_{2^k}(Z[a'][:])               (natural-order butterflies in LDS)
//   scale, codes from U (gamma = 1/sqrt(d_e) folded into the scale).
#include "pme_internal.h"

namespace pme {
namespace {

constexpr int kThreads = 256;

template <typename T> __device__ __forceinline__ float load_as_float(const T* p);
template <> __device__ __forceinline__ float load_as_float<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_as_float<uint16_t>(const uint16_t* p) {
    return __uint_as_float(((uint32_t)*p) << 16);   // bf16 -> fp32 is exact
}

__device__ __forceinline__ float block_reduce(float v, float* red, bool want_max) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int off = 32; off > 0; off >>= 1) {
        float o = __shfl_xor(v, off);
        v = want_max ? fmaxf(v, o) : fminf(v, o);
    }
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
    for (int w = 1; w < kThreads / 64; ++w) r = want_max ? fmaxf(r, red[w]) : fminf(r, red[w]);
    return r;
}

template <typename InT>
__global__ void __launch_bounds__(kThreads)
k_rotate_generic(const InT* __restrict__ x, int64_t ldx, int d, int d_e, int b, int k,
                 double gamma, uint8_t* __restrict__ qx, float* __restrict__ sx,
                 int32_t* __restrict__ zx, uint8_t* __restrict__ ex, float* __restrict__ xhat) {
    extern __shared__ __align__(16) float smem[];
    float* buf = smem;                                            // d_e floats
    float* red = smem + d_e;                                      // 8 floats
    signed char* chi = reinterpret_cast<signed char*>(red + 8);   // q entries
    const int tid = threadIdx.x;
    const int64_t t = blockIdx.x;
    const int n = 1 << k;
    const int q = b - 1;
    const InT* xr = x + t * ldx;

    if (b > 1) fill_quadratic_character(chi, q, tid, kThreads);

    const int rows = (d + n - 1) >> k;   // base rows that hold at least one real input
    for (int idx = tid; idx < d_e; idx += kThreads) {
        const int ap = idx >> k, c = idx & (n - 1);
        float z = 0.f;
        for (int a = 0; a < rows; ++a) {
            const int i = (a << k) + c;
            if (i < d) {
                const float v = load_as_float(xr + i);
                const int sgn = (b > 1) ? paley_entry(chi, q, a, ap) : 1;
                z += (sgn > 0) ? v : -v;
            }
        }
        buf[idx] = z;
    }
    __syncthreads();

    for (int s = 0; s < k; ++s) {
        const int h = 1 << s;
        for (int p = tid; p < d_e / 2; p += kThreads) {
            const int j = ((p >> s) << (s + 1)) | (p & (h - 1));
            const float u = buf[j], v = buf[j + h];
            buf[j] = u + v;
            buf[j + h] = u - v;
        }
        __syncthreads();
    }

    if (xhat) {
        const float g = (float)gamma;
        for (int idx = tid; idx < d_e; idx += kThreads) xhat[t * d_e + idx] = buf[idx] * g;
    }
    if (!qx) return;

    if (ex) {
        // MXFP4 (OCP MX: E8M0 scale per 32 elements, E2M1 elements, round half to even, saturating)
        const float g = (float)gamma;
        for (int blk = tid; blk < d_e / 32; blk += kThreads) {
            float amax = 0.f;
            for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(buf[blk * 32 + i] * g));
            const uint32_t byte = mx_scale_byte(amax);
            const float X = mx_scale_value(byte);
            uint32_t* out = reinterpret_cast<uint32_t*>(qx + t * (int64_t)(d_e / 2) + blk * 16);
            for (int wd = 0; wd < 4; ++wd) {
                const float* bp = buf + blk * 32 + wd * 8;
                const uint32_t word = mx_pack8(bp[0] * g, bp[1] * g, bp[2] * g, bp[3] * g, bp[4] * g, bp[5] * g,
                                               bp[6] * g, bp[7] * g, X);
                out[wd] = word;
            }
            ex[t * (int64_t)(d_e / 32) + blk] = (uint8_t)byte;
        }
        return;
    }

    if (!zx) {
        float m = 0.f;
        for (int idx = tid; idx < d_e; idx += kThreads) m = fmaxf(m, fabsf(buf[idx]));
        m = block_reduce(m, red, true);
        float s = 1.f, rinv = 0.f;
        if (m > 0.f) {
            s = (float)((double)m * gamma / 7.0);
            rinv = (float)(gamma / (double)s);
        }
        if (tid == 0) sx[t] = s;
        uint8_t* out = qx + t * (int64_t)(d_e / 2);
        for (int p = tid; p < d_e / 2; p += kThreads) {
            int q0 = (int)rintf(buf[2 * p] * rinv), q1 = (int)rintf(buf[2 * p + 1] * rinv);
            q0 = min(7, max(-8, q0));
            q1 = min(7, max(-8, q1));
            out[p] = (uint8_t)((q0 & 0xF) | ((q1 & 0xF) << 4));
        }
    } else {
        float lo = 0.f, hi = 0.f;
        for (int idx = tid; idx < d_e; idx += kThreads) {
            lo = fminf(lo, buf[idx]);
            hi = fmaxf(hi, buf[idx]);
        }
        lo = block_reduce(lo, red, false);
        hi = block_reduce(hi, red, true);
        float s = 1.f, rinv = 0.f;
        int z = 0;
        if (hi > lo) {
            s = (float)(((double)hi - (double)lo) * gamma / 15.0);
            rinv = (float)(gamma / (double)s);
            z = (int)rint(-(double)lo * gamma / (double)s);
            z = min(15, max(0, z));
        }
        if (tid == 0) { sx[t] = s; zx[t] = z; }
        uint8_t* out = qx + t * (int64_t)(d_e / 2);
        for (int p = tid; p < d_e / 2; p += kThreads) {
            int q0 = (int)rintf(buf[2 * p] * rinv) + z, q1 = (int)rintf(buf[2 * p + 1] * rinv) + z;
            q0 = min(15, max(0, q0));
            q1 = min(15, max(0, q1));
            out[p] = (uint8_t)(q0 | (q1 << 4));
        }
    }
}

}  // namespace

pme_status launch_rotate_generic(const RotateArgs& a) {
    const size_t lds = (size_t)a.d_e * 4 + 8 * 4 + 512;      // token as fp32, reduction scratch, quadratic characters (q <= 311)
    if (lds > 160 * 1024) return PME_ERR_UNSUPPORTED_PATH;
    if (a.dry) return PME_OK;
    const double gamma = 1.0 / sqrt((double)a.d_e);
    // the attribute is set once per kernel and device, to the largest size accepted above
    static std::atomic<uint32_t> done[2];
    if (a.xt == PME_F32) {
        auto kern = k_rotate_generic<float>;
        if (lds > 64 * 1024 && allow_dynamic_lds(kern, 160 * 1024, done[0]) != PME_OK) return PME_ERR_HIP;
        hipLaunchKernelGGL(kern, dim3((unsigned)a.T), dim3(kThreads), lds, a.stream,
                           (const float*)a.x, a.ldx, (int)a.d, (int)a.d_e, a.b, a.k, gamma,
                           a.qx, a.sx, a.zx, a.ex, a.xhat);
    } else {
        auto kern = k_rotate_generic<uint16_t>;
        if (lds > 64 * 1024 && allow_dynamic_lds(kern, 160 * 1024, done[1]) != PME_OK) return PME_ERR_HIP;
        hipLaunchKernelGGL(kern, dim3((unsigned)a.T), dim3(kThreads), lds, a.stream,
                           (const uint16_t*)a.x, a.ldx, (int)a.d, (int)a.d_e, a.b, a.k, gamma,
                           a.qx, a.sx, a.zx, a.ex, a.xhat);
    }
    return hip_status(hipGetLastError());
}

}  // namespace pme
