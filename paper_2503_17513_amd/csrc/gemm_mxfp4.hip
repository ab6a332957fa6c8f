// MXFP4 x MXFP4 GEMM (the paper's second quantization setting, Section 4: OCP MXFP4 for weights and
// activations, one E8M0 scale per 32 elements) on the block-scaled FP4 matrix instruction of gfx950:
//
//   y[t][n] = bf16( sum over blocks of 32 of 2^(ex - 127) 2^(ew - 127) sum_i P_x,i P_w,i ).
//
// v_mfma_scale_f32_32x32x64_f8f6f4 takes 32 E2M1 codes per lane (one MX block: 16 bytes, exactly what
// one ds_read_b128 brings) and one E8M0 byte per lane for each operand, so nothing is unpacked: packed
// codes and scale bytes travel HBM -> LDS by DMA (same staged ring as the int4 kernel) and LDS -> MFMA.
// Accumulation is fp32 in the matrix core; the epilogue rounds to bf16 and stores 16-byte row pieces.
#include "pme_internal.h"

#include <algorithm>
#include <cstdio>
#include <string>
#include <type_traits>
#include <utility>

namespace pme {
namespace {

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

#define PME_AS3 __attribute__((address_space(3)))

template <int RB> __device__ __forceinline__ int swz(int r) {
    return RB == 64 ? (((r >> 2) ^ r) & 3) : (r & 7);
}
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
// DMA of 16 / 4 bytes per lane into LDS at lds_base + 16 / 4 * lane (lds_base wave-uniform).  Overwrites M0,
// which the compiler does not keep values in; nothing else in this kernel makes the compiler use M0.
// The source is a wave-uniform 64-bit base (SGPR pair) plus a 32-bit byte offset per lane.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}
__device__ __forceinline__ void dma4(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    const bf16x2 p = __builtin_convertvector(f32x2{a, b}, bf16x2);
    return __builtin_bit_cast(uint32_t, p);
}

// BM x BN output tile, WGM x WGN waves, RB packed bytes (2 RB codes, RB / 16 scale bytes) per row and K step.
// LOADER: one more wave per workgroup issues every DMA (codes and scale bytes of every stage) and waits for them;
// the matrix waves issue none (as in the int4 kernel: issuing a DMA holds a wave up for tens of cycles).
template <int BM, int BN, int WGM, int WGN, int RB, int NSTAGE, bool LOADER = false>
__global__ void __launch_bounds__(64 * (WGM * WGN + (LOADER ? 1 : 0)))
k_mxgemm_mfma(const uint8_t* __restrict__ qx, const uint8_t* __restrict__ ex, const uint8_t* __restrict__ qw,
              const uint8_t* __restrict__ ew, int T, int N, int kb, int eb, uint16_t* __restrict__ y, int64_t ldo,
              int tiles_m, int tiles_n, int xcd_gm, int vec_store) {
    constexpr int NW = WGM * WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN, FM = WM / 32, FN = WN / 32;
    constexpr int ROWS = BM + BN;
    constexpr int CPR = RB / 16, RPB = 64 / CPR, BLKS = ROWS / RPB;
    constexpr int CH = (BLKS + NW - 1) / NW;          // code DMA instructions per wave per stage
    constexpr int SW = RB / 64;                       // scale dwords per row per K step
    constexpr int SBLKS = (ROWS / 64) * SW;           // scale DMA blocks (64 rows x 4 bytes) per stage
    constexpr int SCH = (SBLKS + NW - 1) / NW;        // scale DMA instructions per wave per stage
    constexpr int CODE_BYTES = ROWS * RB;
    constexpr int STAGE = CODE_BYTES + ROWS * 4 * SW;
    constexpr int NSUB = RB / 32;                     // MFMA K steps (64 codes) per K step
    constexpr int SLAB = 32 * WN * 2;
    static_assert(ROWS % 64 == 0, "scale DMA moves 64 rows at a time");
    static_assert(NW * SLAB <= NSTAGE * STAGE, "epilogue staging must fit in the K-loop stages");

    extern __shared__ __align__(1024) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    int tm, tn;
    xcd_tile((int)blockIdx.x, tiles_m, tiles_n, xcd_gm, tm, tn);     // compact tile block per XCD
    const int m0 = tm * BM, n0 = tn * BN;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(PME_AS3 unsigned char*)smem;
    const int KT = kb / RB;
    if constexpr (LOADER) {
        if (wave == NW) {
            // The loader wave meets the matrix waves at their barriers (one before the K loop, one per K step, one
            // after the loop) and leaves after the last; later barriers count the waves still running.
            static_assert(RPB % (RB == 64 ? 16 : 8) == 0, "the swizzle must not depend on the block");
            constexpr int PER_STAGE = BLKS + SBLKS;
            constexpr int FIRST_WAIT = (NSTAGE - 1) * PER_STAGE < 63 ? (NSTAGE - 1) * PER_STAGE : 63;   // vmcnt has 6 bits
            static_assert((NSTAGE - 2) * PER_STAGE <= 63, "the wait count of the K loop must fit vmcnt");
            const int lr = lane / CPR, kc = (lane % CPR) ^ swz<RB>(lr);
            uint32_t off[BLKS], soff[SBLKS];
#pragma unroll
            for (int blk = 0; blk < BLKS; ++blk) {
                const int r = RPB * blk + lr;
                const int row = (r < BM) ? min(m0 + r, T - 1) : min(n0 + r - BM, N - 1);
                off[blk] = (uint32_t)row * (uint32_t)kb + (uint32_t)(kc * 16);
            }
#pragma unroll
            for (int sb = 0; sb < SBLKS; ++sb) {
                const int plane = sb / (ROWS / 64), r = 64 * (sb % (ROWS / 64)) + lane;
                const int row = (r < BM) ? min(m0 + r, T - 1) : min(n0 + r - BM, N - 1);
                soff[sb] = (uint32_t)row * (uint32_t)eb + (uint32_t)(4 * plane);
            }
            auto issue_stage = [&](int stage, int kt) {
                const uint8_t* pa = qx + (int64_t)kt * RB;
                const uint8_t* pb = qw + (int64_t)kt * RB;
                const uint8_t* sa = ex + (int64_t)kt * (RB / 16);
                const uint8_t* sb_ = ew + (int64_t)kt * (RB / 16);
#pragma unroll
                for (int blk = 0; blk < BLKS; ++blk)
                    dma16(blk < BM / RPB ? pa : pb, off[blk], lds0 + stage * STAGE + blk * 1024);
#pragma unroll
                for (int sb = 0; sb < SBLKS; ++sb)
                    dma4(64 * (sb % (ROWS / 64)) < BM ? sa : sb_, soff[sb], lds0 + stage * STAGE + CODE_BYTES + sb * 256);
            };
#pragma unroll
            for (int st = 0; st < NSTAGE; ++st) issue_stage(st, min(st, KT - 1));
            wait_vm<FIRST_WAIT>();
            lds_barrier();
            int cur = 0;
            for (int kt = 0; kt + 1 < KT; ++kt) {
                wait_vm<(NSTAGE - 2) * PER_STAGE>();
                lds_barrier();          // K step kt + 1 has landed; every wave has left the stage of K step kt
                issue_stage(cur, min(kt + NSTAGE, KT - 1));
                cur = (cur == NSTAGE - 1) ? 0 : cur + 1;
            }
            wait_vm<0>();
            lds_barrier();
            return;
        }
    }

    // A DMA block lies wholly in the token rows or wholly in the channel rows, so the operand a slot reads
    // from is wave-uniform; the lane keeps its byte offset within that operand.
    static_assert(BM % RPB == 0 && BM % 64 == 0, "DMA blocks do not straddle the operands");
    uint32_t voff[CH];
#pragma unroll
    for (int s = 0; s < CH; ++s) {
        const int r = RPB * ((wave + NW * s) % BLKS) + lane / CPR;
        const int kc = (lane % CPR) ^ swz<RB>(r);
        const int row = (r < BM) ? min(m0 + r, T - 1) : min(n0 + r - BM, N - 1);
        voff[s] = (uint32_t)row * (uint32_t)kb + (uint32_t)(kc * 16);
    }
    // scale bytes: block sb = plane * (ROWS / 64) + rows-of-64 index; lane = row within the 64
    uint32_t svoff[SCH];
#pragma unroll
    for (int s = 0; s < SCH; ++s) {
        const int sb = (wave + NW * s) % SBLKS;
        const int plane = sb / (ROWS / 64), r = 64 * (sb % (ROWS / 64)) + lane;
        const int row = (r < BM) ? min(m0 + r, T - 1) : min(n0 + r - BM, N - 1);
        svoff[s] = (uint32_t)row * (uint32_t)eb + (uint32_t)(4 * plane);
    }
    // DMA slot q of this wave for K step kt: slots 0 .. CH - 1 move codes, CH .. CH + SCH - 1 scale bytes
    constexpr int NSLOT = CH + SCH;
    auto issue_slot = [&](int stage, int kt, int q) {
        if (q < CH) {
            const int blk = (wave + NW * q) % BLKS;
            dma16((blk < BM / RPB ? qx : qw) + (int64_t)kt * RB, voff[q], lds0 + stage * STAGE + blk * 1024);
        } else {
            const int sb = (wave + NW * (q - CH)) % SBLKS;
            dma4((64 * (sb % (ROWS / 64)) < BM ? ex : ew) + (int64_t)kt * (RB / 16), svoff[q - CH],
                 lds0 + stage * STAGE + CODE_BYTES + sb * 256);
        }
    };
    auto issue = [&](int stage, int kt) {
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) issue_slot(stage, kt, q);
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int frow = lane & 31, fk = lane >> 5;
    int aoff[FM], boff[FN], asoff[FM], bsoff[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int r = wm * WM + 32 * i + frow;
        aoff[i] = r * RB + ((fk ^ swz<RB>(r)) << 4);
        asoff[i] = CODE_BYTES + r * 4;
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int r = BM + wn * WN + 32 * j + frow;
        boff[j] = r * RB + ((fk ^ swz<RB>(r)) << 4);
        bsoff[j] = CODE_BYTES + r * 4;
    }
    struct Frags { u32x4 a[FM], b[FN]; uint32_t sa[FM], sb[FN]; };
    // sub-step s: codes of block 2 s + fk of the row (chunk position (2 s + fk) ^ swz), and its scale: byte
    // (2 s + fk) & 3 of scale dword (2 s + fk) >> 2 = s >> 1.  The dword is read once per pair of sub-steps
    // and shifted by 8 fk bits, which puts the scale of the even sub-step in byte 0 and of the odd one in
    // byte 2; the matrix instruction picks the byte (its scale operand select), so the odd sub-step takes
    // the register of the even one (`even`) and reads nothing.
    auto load_frags = [&](Frags& f, const unsigned char* stage, int s, const Frags& even) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            f.a[i] = *reinterpret_cast<const u32x4*>(stage + (aoff[i] ^ (s << 5)));
            if (s & 1) f.sa[i] = even.sa[i];
            else f.sa[i] = *reinterpret_cast<const uint32_t*>(stage + asoff[i] + (s >> 1) * ROWS * 4) >> (8 * fk);
        }
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            f.b[j] = *reinterpret_cast<const u32x4*>(stage + (boff[j] ^ (s << 5)));
            if (s & 1) f.sb[j] = even.sb[j];
            else f.sb[j] = *reinterpret_cast<const uint32_t*>(stage + bsoff[j] + (s >> 1) * ROWS * 4) >> (8 * fk);
        }
    };
    // formats 4 = FP4 E2M1 for both operands; odd: the sub-step's scales sit in byte 2 of the scale registers
    auto mfma_ij = [&](const Frags& f, int i, int j, bool odd) {
        const i32x8 xa = {(int)f.a[i][0], (int)f.a[i][1], (int)f.a[i][2], (int)f.a[i][3], 0, 0, 0, 0};
        const i32x8 wb = {(int)f.b[j][0], (int)f.b[j][1], (int)f.b[j][2], (int)f.b[j][3], 0, 0, 0, 0};
        if (odd)
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wb, xa, acc[i][j], 4, 4, 2, (int)f.sb[j], 2,
                                                                        (int)f.sa[i]);
        else
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wb, xa, acc[i][j], 4, 4, 0, (int)f.sb[j], 0,
                                                                        (int)f.sa[i]);
    };
    auto mfma_one = [&](const Frags& f, auto mc, bool odd) {  // instruction m of the FM x FN of a sub-step
        mfma_ij(f, decltype(mc)::value / FN, decltype(mc)::value % FN, odd);
    };
    auto mfma_all = [&](const Frags& f, bool odd) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) mfma_ij(f, i, j, odd);
    };

    // Pipeline over sub-steps g = kt NSUB + s: read the fragments of g + 1 while the matrix cores work on g.
    // Before the region whose read first touches K step kt + 1 (s = NSUB - 1) every read of K step kt has been
    // issued: wait for the DMA of kt + 1, barrier, start the DMA of kt + NSTAGE into the stage just left.
    if constexpr (!LOADER) {
#pragma unroll
        for (int st = 0; st < NSTAGE; ++st) issue(st, min(st, KT - 1));
        wait_vm<(NSTAGE - 1) * (CH + SCH)>();
    }
    lds_barrier();
    Frags raw[2];
    load_frags(raw[0], smem, 0, raw[0]);
    int cur = 0;
    for (int kt = 0; kt + 1 < KT; ++kt) {
        const int nxt = (cur == NSTAGE - 1) ? 0 : cur + 1;
        const unsigned char* scur = smem + cur * STAGE;
        const unsigned char* snxt = smem + nxt * STAGE;
#pragma unroll
        for (int s = 0; s < NSUB; ++s) {
            if (LOADER && s == NSUB - 1) {
                lds_barrier();
                load_frags(raw[(s + 1) & 1], snxt, 0, raw[s & 1]);
                mfma_all(raw[s & 1], (s & 1) != 0);
            } else if (s == NSUB - 1) {
                wait_vm<(NSTAGE - 2) * (CH + SCH)>();
                lds_barrier();
                load_frags(raw[(s + 1) & 1], snxt, 0, raw[s & 1]);
                // refill the stage just left with K step kt + NSTAGE: the DMA instructions go between the
                // matrix instructions, which keep the pipe busy while the wave is held up issuing them
                const int ktn = min(kt + NSTAGE, KT - 1);
                constexpr int NM = FM * FN;
                constexpr int NP = NM < NSLOT ? NM : NSLOT;
                static_for<NP>([&](auto pc) {
                    constexpr int c = decltype(pc)::value;
                    static_for<NM>([&](auto mc) {
                        if constexpr (decltype(mc)::value * NP / NM == c) mfma_one(raw[s & 1], mc, (s & 1) != 0);
                    });
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<NSLOT>([&](auto qc) {
                        if constexpr (decltype(qc)::value * NP / NSLOT == c) issue_slot(cur, ktn, decltype(qc)::value);
                    });
                    __builtin_amdgcn_sched_barrier(0);
                });
            } else {
                load_frags(raw[(s + 1) & 1], scur, s + 1, raw[s & 1]);
                mfma_all(raw[s & 1], (s & 1) != 0);
            }
        }
        cur = nxt;
    }
    {
        const unsigned char* scur = smem + cur * STAGE;
#pragma unroll
        for (int s = 0; s < NSUB; ++s) {
            if (s + 1 < NSUB) load_frags(raw[(s + 1) & 1], scur, s + 1, raw[s & 1]);
            mfma_all(raw[s & 1], (s & 1) != 0);
        }
    }
    if constexpr (!LOADER) wait_vm<0>();
    lds_barrier();

    // ---- epilogue.  Accumulator element e of block (i, j): output channel n0 + wn WN + 32 j + 8 (e / 4) + 4 fk + e % 4,
    // token m0 + wm WM + 32 i + frow.  One 32-token slab at a time goes through LDS (private to the wave).
    unsigned char* slab = smem + (size_t)wave * SLAB;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int eg = 0; eg < 4; ++eg) {
                const u32x2 pk = u32x2{pack_bf16(acc[i][j][4 * eg], acc[i][j][4 * eg + 1]),
                                       pack_bf16(acc[i][j][4 * eg + 2], acc[i][j][4 * eg + 3])};
                *reinterpret_cast<u32x2*>(slab + frow * (WN * 2) + (32 * j + 8 * eg + 4 * fk) * 2) = pk;
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        const int tbase = m0 + wm * WM + 32 * i, nbase = n0 + wn * WN;
        if (vec_store) {
            constexpr int CPS = WN / 8;
#pragma unroll
            for (int c = lane; c < 32 * CPS; c += 64) {
                const int row = c / CPS, col = (c % CPS) * 8;
                const u32x4 v = *reinterpret_cast<const u32x4*>(slab + row * (WN * 2) + col * 2);
                if (tbase + row < T && nbase + col < N)
                    *reinterpret_cast<u32x4*>(y + (int64_t)(tbase + row) * ldo + nbase + col) = v;
            }
        } else {
            for (int c = lane; c < 32 * WN; c += 64) {
                const int row = c / WN, col = c % WN;
                if (tbase + row < T && nbase + col < N)
                    y[(int64_t)(tbase + row) * ldo + nbase + col] = *reinterpret_cast<const uint16_t*>(slab + row * (WN * 2) + col * 2);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
}

template <int BM, int BN, int WGM, int WGN, int RB, int NSTAGE, bool LOADER = false>
pme_status launch_tile(const MxGemmArgs& a) {
    const int kb = (int)(a.d_e / 2), eb = (int)(a.d_e / 32);
    if (kb % RB) return PME_ERR_UNSUPPORTED_PATH;
    if ((int64_t)std::max(a.T, a.N) * kb >= (int64_t(1) << 32)) return PME_ERR_UNSUPPORTED_PATH;   // 32-bit DMA offsets
    if (a.dry) {
        if (a.plan) {
            // the instantiation's name as a profiler prints it
            static const std::string name = [] {
                char buf[96];
                snprintf(buf, sizeof buf, "k_mxgemm_mfma<%d, %d, %d, %d, %d, %d, %s>", BM, BN, WGM, WGN, RB, NSTAGE, LOADER ? "true" : "false");
                return std::string(buf);
            }();
            *a.plan = name.c_str();
        }
        return PME_OK;
    }
    const int tiles_m = (int)((a.T + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(64 * (WGM * WGN + (LOADER ? 1 : 0)));
    const size_t lds = (size_t)NSTAGE * ((BM + BN) * RB + (BM + BN) * 4 * (RB / 64));
    auto kern = k_mxgemm_mfma<BM, BN, WGM, WGN, RB, NSTAGE, LOADER>;
    static std::atomic<uint32_t> done;
    if (lds > 64 * 1024 && allow_dynamic_lds(kern, (int)lds, done) != PME_OK) return PME_ERR_HIP;
    const int vec = (a.N % 8 == 0 && a.ldy % 8 == 0 && (reinterpret_cast<uintptr_t>(a.y) & 15) == 0) ? 1 : 0;
    hipLaunchKernelGGL(kern, grid, block, lds, a.stream, a.qx, a.ex, a.qw, a.ew, (int)a.T, (int)a.N, kb, eb,
                       static_cast<uint16_t*>(a.y), a.ldy, tiles_m, tiles_n, xcd_grid_m(tiles_m, tiles_n, BM, BN), vec);
    return hip_status(hipGetLastError());
}

// Plain-ALU MXFP4 GEMM, one thread per output: every shape, and the cross-check of the MFMA kernel.
__device__ __forceinline__ float e2m1_value(uint32_t c) {
    const uint32_t E = (c >> 1) & 3u, M = c & 1u;
    const float mag = E == 0 ? 0.5f * (float)M : (1.f + 0.5f * (float)M) * (float)(1u << (E - 1));
    return (c & 8u) ? -mag : mag;
}
__global__ void __launch_bounds__(256)
k_mxgemm_generic(const uint8_t* __restrict__ qx, const uint8_t* __restrict__ ex, const uint8_t* __restrict__ qw,
                 const uint8_t* __restrict__ ew, int T, int N, int d_e, uint16_t* __restrict__ y, int64_t ldo) {
    const int n = blockIdx.x * 16 + (threadIdx.x & 15);
    if (n >= N) return;
    const uint8_t* wr = qw + (int64_t)n * (d_e / 2);
    // blocks of 16 tokens: the grid's y extent is capped (65535), so a workgroup walks its share of them
    for (int64_t t = (int64_t)blockIdx.y * 16 + (threadIdx.x >> 4); t < T; t += (int64_t)gridDim.y * 16) {
        const uint8_t* ar = qx + t * (d_e / 2);
        double sum = 0.0;
        for (int blk = 0; blk < d_e / 32; ++blk) {
            float inner = 0.f;      // exact: multiples of 1/4 bounded by 32 * 36
            for (int p = 0; p < 16; ++p) {
                const uint32_t av = ar[blk * 16 + p], wv = wr[blk * 16 + p];
                inner += e2m1_value(av & 0xF) * e2m1_value(wv & 0xF) + e2m1_value(av >> 4) * e2m1_value(wv >> 4);
            }
            const int e = (int)ex[t * (d_e / 32) + blk] + (int)ew[(int64_t)n * (d_e / 32) + blk] - 254;
            sum += ldexp((double)inner, e);
        }
        y[t * ldo + n] = f32_to_bf16_bits((float)sum);
    }
}

int g_mx_tile_override = 0;

// ---- few tokens (at most 32): memory-bound on the packed weights, like the int4 decode kernel.  One workgroup
// owns 16 output channels and all of K; its waves split K into runs of 64-byte chunks (128 codes = 4 MX blocks),
// every weight byte is loaded once into registers.  A chunk of 16 channels is one 16-byte load per lane (lane =
// channel % 16 + 16 * block of the chunk) plus that block's scale byte, and feeds
// v_mfma_scale_f32_16x16x128_f8f6f4 against the token chunks of up to TG groups of 16 tokens.  The waves'
// partial 16 x 16 tiles (fp32) are summed through LDS.
typedef __attribute__((ext_vector_type(4))) float f32x4;

// KB: chunks a wave keeps in flight at once (its share of K in one round of loads where that fits in 8).
template <int NW, int TG, int KB>
__global__ void __launch_bounds__(64 * NW)
k_mxgemm_decode(const uint8_t* __restrict__ qx, const uint8_t* __restrict__ ex, const uint8_t* __restrict__ qw,
                const uint8_t* __restrict__ ew, int T, int N, int kb, int eb, uint16_t* __restrict__ y, int64_t ldo) {
    __shared__ float part[NW][64][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, kg = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int nchunks = kb >> 6;
    const int c0 = (int)(((int64_t)wave * nchunks) / NW), c1 = (int)(((int64_t)(wave + 1) * nchunks) / NW);
    const int64_t wr = min(n0 + r, N - 1);
    const uint8_t* wrow = qw + wr * kb + kg * 16;
    const uint8_t* wsrow = ew + wr * eb + kg;
    const uint8_t* xrow[TG];
    const uint8_t* xsrow[TG];
#pragma unroll
    for (int g = 0; g < TG; ++g) {
        const int64_t xr = min(16 * g + r, T - 1);
        xrow[g] = qx + xr * kb + kg * 16;
        xsrow[g] = ex + xr * eb + kg;
    }
    f32x4 acc[TG];
#pragma unroll
    for (int g = 0; g < TG; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int c = c0; c < c1; c += KB) {
        u32x4 w[KB], x[TG][KB];
        uint32_t ws[KB], xs[TG][KB];
#pragma unroll
        for (int i = 0; i < KB; ++i) {
            if (c + i < c1) {                           // wave-uniform: surplus slots load nothing
                const int cc = c + i;
                w[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wrow + (int64_t)cc * 64));
                ws[i] = wsrow[cc * 4];
#pragma unroll
                for (int g = 0; g < TG; ++g) {
                    x[g][i] = *reinterpret_cast<const u32x4*>(xrow[g] + (int64_t)cc * 64);
                    xs[g][i] = xsrow[g][cc * 4];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < KB; ++i) {
            if (c + i < c1) {
                const i32x8 wb = {(int)w[i][0], (int)w[i][1], (int)w[i][2], (int)w[i][3], 0, 0, 0, 0};
#pragma unroll
                for (int g = 0; g < TG; ++g) {
                    const i32x8 xa = {(int)x[g][i][0], (int)x[g][i][1], (int)x[g][i][2], (int)x[g][i][3], 0, 0, 0, 0};
                    acc[g] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(wb, xa, acc[g], 4, 4, 0, (int)ws[i], 0,
                                                                               (int)xs[g][i]);
                }
            }
        }
    }
#pragma unroll
    for (int g = 0; g < TG; ++g) {
        if (g > 0) __syncthreads();                     // the previous group has been read
#pragma unroll
        for (int i = 0; i < 4; ++i) part[wave][lane][i] = acc[g][i];
        __syncthreads();
        if (tid < 256) {
            // element tid = 4 * lane' + i of the 16 x 16 tile: channel 4 * (lane' / 16) + i, token lane' % 16
            const int ln = tid >> 2, i = tid & 3;
            float sum = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2) sum += part[w2][ln][i];
            const int t = 16 * g + (ln & 15), n = n0 + 4 * (ln >> 4) + i;
            if (t < T && n < N) y[(int64_t)t * ldo + n] = f32_to_bf16_bits(sum);
        }
    }
}

template <int NW, int TG, int KB>
pme_status launch_mx_decode_kb(const MxGemmArgs& a) {
    hipLaunchKernelGGL((k_mxgemm_decode<NW, TG, KB>), dim3((unsigned)((a.N + 15) / 16)), dim3(64 * NW), 0, a.stream, a.qx,
                       a.ex, a.qw, a.ew, (int)a.T, (int)a.N, (int)(a.d_e / 2), (int)(a.d_e / 32),
                       static_cast<uint16_t*>(a.y), a.ldy);
    return hip_status(hipGetLastError());
}
template <int NW, int TG>
pme_status launch_mx_decode_nw(const MxGemmArgs& a) {
    // (two token groups on 16 waves have 128 registers per lane: 4 chunks)
    const int64_t per_wave = (a.d_e / 128 + NW - 1) / NW;
    if constexpr (TG > 1 && NW == 16) {
        return launch_mx_decode_kb<NW, TG, 4>(a);
    } else {
        if (per_wave <= 4) return launch_mx_decode_kb<NW, TG, 4>(a);
        if (per_wave <= 6) return launch_mx_decode_kb<NW, TG, 6>(a);
        return launch_mx_decode_kb<NW, TG, 8>(a);
    }
}
template <int TG>
pme_status launch_mx_decode_groups(const MxGemmArgs& a) {
    const int64_t nchunks = a.d_e / 128;
    if (nchunks >= 32) return launch_mx_decode_nw<16, TG>(a);
    if (nchunks >= 8) return launch_mx_decode_nw<8, TG>(a);
    return launch_mx_decode_nw<4, TG>(a);
}

}  // namespace

void set_mxgemm_tile_override(int id) { g_mx_tile_override = id; }

pme_status launch_mxgemm_generic(const MxGemmArgs& a) {
    if (a.dry) {
        if (a.plan) *a.plan = "k_mxgemm_generic";
        return PME_OK;
    }
    dim3 grid((unsigned)((a.N + 15) / 16), (unsigned)std::min<int64_t>((a.T + 15) / 16, 65535));
    hipLaunchKernelGGL(k_mxgemm_generic, grid, dim3(256), 0, a.stream, a.qx, a.ex, a.qw, a.ew, (int)a.T, (int)a.N,
                       (int)a.d_e, static_cast<uint16_t*>(a.y), a.ldy);
    return hip_status(hipGetLastError());
}

pme_status launch_mxgemm_decode(const MxGemmArgs& a) {
    // at most 32 tokens (beyond that the tiled kernel measured faster), whole 64-byte chunks, 16-byte aligned code rows
    if (a.T > 32 || a.d_e % 128 || a.d_e > (1 << 20)) return PME_ERR_UNSUPPORTED_PATH;
    if ((reinterpret_cast<uintptr_t>(a.qx) & 15) || (reinterpret_cast<uintptr_t>(a.qw) & 15)) return PME_ERR_UNSUPPORTED_PATH;
    if (a.dry) {
        if (a.plan) *a.plan = "k_mxgemm_decode";
        return PME_OK;
    }
    if (a.T <= 16) return launch_mx_decode_groups<1>(a);
    return launch_mx_decode_groups<2>(a);
}

pme_status launch_mxgemm_mfma(const MxGemmArgs& a) {
    // whole 64-byte K steps (d_e % 128 == 0: also makes the scale rows 4-byte aligned), 16-byte aligned code rows
    if (a.d_e % 128 || a.d_e > (1 << 20)) return PME_ERR_UNSUPPORTED_PATH;
    if ((reinterpret_cast<uintptr_t>(a.qx) & 15) || (reinterpret_cast<uintptr_t>(a.qw) & 15) ||
        (reinterpret_cast<uintptr_t>(a.ex) & 3) || (reinterpret_cast<uintptr_t>(a.ew) & 3))
        return PME_ERR_UNSUPPORTED_PATH;
    const int64_t cus = 256;
    auto tiles = [&](int bm, int bn) { return ((a.T + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
    int id = g_mx_tile_override;
    if (id == 0) {
        const bool wide = (a.d_e % 256) == 0;
        if (tiles(128, 128) >= cus / 2) {
            // The cheapest of four tile shapes by rounds x tile area / efficiency, as in the int4 kernel.  With FP4
            // the small tiles are far less efficient (their LDS traffic per matrix instruction is the bound), so
            // 256 x 256 pays from about half of the compute units on.  Efficiencies relative to 256 x 256 and the
            // cost of sharing a compute unit are fitted to a sweep of every tile over 12 outputs, whose fastest
            // tile the model names in each.
            auto rounds = [&](int64_t t) { return (double)((t + cus - 1) / cus); };
            auto rounds_shared = [&](int64_t t) {          // two workgroups may share a compute unit
                const int64_t pairs = (t - 1) / (2 * cus);
                const double rest = (double)(t - 2 * cus * pairs) / (double)cus;       // (0, 2]
                return 1.7 * (double)pairs + (rest <= 1.0 ? 1.0 : 1.5 + 0.2 * (rest - 1.0));
            };
            const double c256 = rounds(tiles(256, 256)) * (256.0 * 256.0) / 1.00;
            const double c9 = wide ? rounds(tiles(256, 128)) * (256.0 * 128.0) / 0.72 : 1e30;     // 128-byte rows only
            const double c192 = rounds_shared(tiles(128, 192)) * (128.0 * 192.0) / 0.55;
            const double c128 = rounds_shared(tiles(128, 128)) * (128.0 * 128.0) / 0.47;
            const double best = std::min(std::min(c256, c9), std::min(c192, c128));
            if (best == c256) id = wide ? 8 : 2;
            else if (best == c9) id = 9;
            else if (best == c192) id = tiles(128, 192) > cus ? 5 : (wide ? 6 : 10);
            else id = wide ? 3 : 4;
        } else {
            id = 11;
        }
    }
    switch (id) {
        case 1: return launch_tile<256, 256, 2, 2, 128, 2>(a);
        case 2: return launch_tile<256, 256, 2, 2, 64, 3>(a);
        case 3: return launch_tile<128, 128, 2, 2, 128, 3>(a);
        case 4: return launch_tile<128, 128, 2, 2, 64, 3>(a);
        case 5: return launch_tile<128, 192, 2, 2, 64, 3>(a);
        case 6: return launch_tile<128, 192, 2, 2, 128, 3>(a);
        case 7: return launch_tile<64, 64, 2, 2, 64, 3>(a);
        case 8: return launch_tile<256, 256, 2, 4, 128, 2>(a);
        case 9: return launch_tile<256, 128, 2, 2, 128, 3>(a);
        // a fifth wave issues all the DMA (pays with 64-byte rows: 128 x 192 -4 %, 64 x 64 up to -14 %; with 128-byte rows
        // at 128 x 128 one wave cannot issue a stage's 40 DMA instructions in the time of its 16 matrix instructions per wave)
        case 10: return launch_tile<128, 192, 2, 2, 64, 3, true>(a);
        case 11: return launch_tile<64, 64, 2, 2, 64, 3, true>(a);
    }
    return PME_ERR_UNSUPPORTED_PATH;
}

}  // namespace pme
