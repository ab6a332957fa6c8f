// W4A4 GEMM on the int8 matrix cores with the dequantising epilogue fused in.
//
//   acc[t][n] = sum_j qx[t][j] qw[n][j]   (paper Section 3: Q(X_hat) Q(W_hat)),
//   y[t][n]   = bf16(acc * sx[t] * sw[n]) (Section 4: per-token and per-channel scales).
//
// Both operands are K-contiguous packed int4.  A workgroup owns a BM x BN output tile and walks K
// in steps of 128 or 256 codes (64 or 128 packed bytes per row).
//  * HBM -> LDS: global_load_lds_dwordx4 (no registers; scalar base + per-lane offset, so no VALU
//    either), two or three LDS stages.  The DMA instructions and the waits on them are issued from
//    inline assembly, so that the compiler does not order LDS reads of one stage after DMA writes
//    to another; the per-step barrier waits for LDS traffic only and for all but the newest
//    stage's DMA (vmcnt counts in order).  The DMA instructions of a K step are spread between the
//    matrix instructions of the region after the barrier (issuing one holds the wave up).
//    In the variants with a loader wave, a fifth wave issues every DMA and the four matrix waves none.
//  * LDS -> registers: one ds_read_b128 per lane brings 32 codes, unpacked in registers into two
//    int8 MFMA operands:   even codes (w & 0x0F0F0F0F) << 4,   odd codes w & 0xF0F0F0F0.
//    A nibble moved to the top of a byte is 16 x its two's-complement value: no sign extension.
//    Both operands carry the factor 16, the int32 accumulator holds 256 x the exact sum
//    (|256 acc| <= 256 * 64 * d_e < 2^31 for d_e < 2^17; at d_e = 2^17 rows of all -8 codes would
//    wrap, so the launcher refuses d_e >= 2^17), removed in the epilogue.  The order in
//    which codes meet inside an MFMA is the same permutation for both operands, which an exact
//    integer sum does not notice.
//  * v_mfma_i32_32x32x32_i8 with the weight fragment as the first operand: a lane then owns one
//    token and runs of four consecutive output channels, which the epilogue scales, rounds to
//    bf16, transposes through LDS and stores as 16-byte row pieces.
#include "pme_internal.h"

#include <algorithm>
#include <cstdio>
#include <string>
#include <type_traits>

namespace pme {
namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

#define PME_AS1 __attribute__((address_space(1)))
#define PME_AS3 __attribute__((address_space(3)))

enum { MODE_BF16 = 0, MODE_ASYM = 1, MODE_I32 = 2 };

// LDS swizzle: the 16-byte chunk kc of tile row r sits at chunk position kc ^ swz(r), so that the rows
// read together by one ds_read_b128 spread over the banks.  RB = bytes per tile row per K step.  The two
// functions are the fastest of the XOR patterns tried on MI355X (timed in the whole kernel, where the
// pattern also decides which global chunk each DMA lane fetches).
template <int RB> __device__ __forceinline__ int swz(int r) {
    return RB == 64 ? (((r >> 2) ^ r) & 3) : (r & 7);
}

// LDS-only barrier: DMA (counted by vmcnt) stays in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base wave-uniform).
// The statement overwrites M0, which the compiler reserves and does not keep values in; no other code in
// this kernel makes the compiler emit an M0 use.
// The source is a wave-uniform 64-bit base (SGPR pair) plus a 32-bit byte offset per lane: no vector
// arithmetic is needed to move the window along K.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    const bf16x2 p = __builtin_convertvector(f32x2{a, b}, bf16x2);     // v_cvt_pk_bf16_f32: round half to even
    return __builtin_bit_cast(uint32_t, p);
}

// BM x BN output tile, WGM x WGN x KS waves, RB packed bytes (2 RB codes) per row and K step, NSTAGE LDS stages.
// KS = 2: two waves share every wave tile and split each K step's sub-steps between them (the first half and
// the second half), so that a compute unit's four waves hold tiles twice as large -- half the fragment reads
// and unpack arithmetic per matrix instruction -- where the output only gives each compute unit a small tile;
// the two partial accumulators are added through LDS before the epilogue.
// LOADER: one more wave per workgroup does nothing but the DMA (all blocks of every stage) and the waits on it; the
// others never issue a DMA.  Issuing a global_load_lds holds a wave up for tens of cycles, during which it starts
// no matrix instruction; a wave of its own takes that off the waves that feed the matrix pipe.
template <int BM, int BN, int WGM, int WGN, int RB, int NSTAGE, int MODE, int KS = 1, bool LOADER = false>
__global__ void __launch_bounds__(64 * (WGM * WGN * KS + (LOADER ? 1 : 0)))
k_gemm_mfma(const uint8_t* __restrict__ qx, const uint8_t* __restrict__ qw,
            const float* __restrict__ sx, const float* __restrict__ sw,
            const int32_t* __restrict__ zx, const int32_t* __restrict__ wsum,
            int T, int N, int kb, void* __restrict__ out, int64_t ldo, int tiles_m, int tiles_n, int xcd_gm, int vec_store) {
    constexpr int NW = WGM * WGN * KS;
    constexpr int WM = BM / WGM, WN = BN / WGN, FM = WM / 32, FN = WN / 32;
    constexpr int ROWS = BM + BN;
    constexpr int CPR = RB / 16;                  // 16-byte chunks per row
    constexpr int RPB = 64 / CPR;                 // rows per 1 KB DMA block
    constexpr int BLKS = ROWS / RPB;              // DMA blocks per stage
    // DMA instructions per wave per stage.  Every wave issues the same number (the per-step wait counts
    // on it); when the blocks do not divide evenly the surplus instructions repeat an earlier block.
    constexpr int CH = (BLKS + NW - 1) / NW;
    constexpr int STAGE = ROWS * RB;
    constexpr int NSUBG = RB / 32;                // sub-steps of 64 codes per K step
    constexpr int NSUB = NSUBG / KS;              // ... of which a wave computes this many
    static_assert(KS == 1 || (KS == 2 && NSUB >= 2 && FM % 2 == 0), "K split: two halves of at least two sub-steps");
    constexpr int XCH = (KS == 2) ? (FM / 2) * FN * 16 * 256 : 0;     // bytes a wave hands to its partner
    static_assert(NW * XCH <= NSTAGE * STAGE, "the partial accumulators are exchanged through the K-loop stages");
    constexpr int SLAB = 32 * WN * 2;             // epilogue: one 32-token slab of the wave tile in bf16
    static_assert(NW * SLAB + ROWS * 8 <= NSTAGE * STAGE, "epilogue staging must fit in the K-loop stages");
    static_assert(NSTAGE == 2 || NSTAGE == 3, "two or three stages");

    extern __shared__ __align__(1024) unsigned char smem[];      // NSTAGE stages

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kh = wave / (WGM * WGN);            // which half of every K step (0 when KS = 1)
    const int wm = (wave % (WGM * WGN)) / WGN, wn = wave % WGN;
    const int s_off = kh * NSUB;                  // first sub-step of this wave within a K step

    int tm, tn;
    xcd_tile((int)blockIdx.x, tiles_m, tiles_n, xcd_gm, tm, tn);     // compact tile block per XCD
    const int m0 = tm * BM, n0 = tn * BN;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(PME_AS3 unsigned char*)smem;
    // K steps: whole steps of RB bytes, the last one possibly half as long (kb is a multiple of 64): its DMA
    // leaves out the chunks beyond the row end and its sub-steps beyond TAIL_SUB are not computed.
    const int KT = (kb + RB - 1) / RB;
    const int tail_chunks = (kb - (KT - 1) * RB) / 16;          // chunks of the last K step
    const int tail_sub = tail_chunks / 2;                       // its sub-steps (64 codes = 2 chunks each)

    if constexpr (LOADER) {
        if (wave == NW) {
            // The loader wave.  It meets the other waves at the same barriers as they meet each other (one before
            // the K loop, one per K step, one after the loop) and leaves after the last of them; later barriers
            // count the waves still running.
            // swz(row) only looks at row bits below RPB's, so a lane moves the same chunk of its row in every block.
            static_assert(RPB % (RB == 64 ? 16 : 8) == 0, "the swizzle must not depend on the block");
            constexpr int FIRST_WAIT = (NSTAGE - 1) * BLKS < 63 ? (NSTAGE - 1) * BLKS : 63;   // vmcnt has 6 bits
            static_assert((NSTAGE - 2) * BLKS <= 63, "the wait count of the K loop must fit vmcnt");
            const int lr = lane / CPR, kc = (lane % CPR) ^ swz<RB>(lr);
            uint32_t off[BLKS];
#pragma unroll
            for (int blk = 0; blk < BLKS; ++blk) {
                const int r = RPB * blk + lr;
                const int row = (r < BM) ? min(m0 + r, T - 1) : min(n0 + r - BM, N - 1);
                off[blk] = (uint32_t)row * (uint32_t)kb + (uint32_t)(kc * 16);
            }
            auto issue_stage = [&](int stage, int kt) {
                const uint8_t* pa = qx + (int64_t)kt * RB;
                const uint8_t* pb = qw + (int64_t)kt * RB;
                if (kt < KT - 1 || kc < tail_chunks) {          // the shortened last K step: lanes beyond the row end idle
#pragma unroll
                    for (int blk = 0; blk < BLKS; ++blk)
                        dma16(blk < BM / RPB ? pa : pb, off[blk], lds0 + stage * STAGE + blk * 1024);
                }
            };
#pragma unroll
            for (int st = 0; st < NSTAGE; ++st) issue_stage(st, min(st, KT - 1));
            wait_vm<FIRST_WAIT>();
            lds_barrier();
            int cur = 0;
            for (int kt = 0; kt + 1 < KT; ++kt) {
                wait_vm<(NSTAGE - 2) * BLKS>();
                lds_barrier();          // K step kt + 1 has landed; every wave has left the stage of K step kt
                issue_stage(cur, min(kt + NSTAGE, KT - 1));
                cur = (cur == NSTAGE - 1) ? 0 : cur + 1;
            }
            wait_vm<0>();
            lds_barrier();
            return;
        }
    }

    // DMA source of each 16-byte chunk this lane moves: block blk covers tile rows RPB blk .. RPB blk + RPB - 1;
    // lane L writes chunk position L % CPR of row RPB blk + L / CPR, which holds chunk (L % CPR) ^ swz(row).
    // A 1 KB block lies wholly in the token rows or wholly in the channel rows (BM is a multiple of RPB), so
    // the operand a DMA slot reads from is wave-uniform; the lane keeps its byte offset within that operand.
    static_assert(BM % RPB == 0, "DMA blocks do not straddle the operands");
    uint32_t voff[CH];
    int kcl[CH];          // logical chunk each DMA slot of this lane carries (for the shortened last K step)
#pragma unroll
    for (int s = 0; s < CH; ++s) {
        const int r = RPB * ((wave + NW * s) % BLKS) + lane / CPR;
        const int kc = (lane % CPR) ^ swz<RB>(r);
        kcl[s] = kc;
        const int row = (r < BM) ? min(m0 + r, T - 1) : min(n0 + r - BM, N - 1);
        voff[s] = (uint32_t)row * (uint32_t)kb + (uint32_t)(kc * 16);
    }
    // The tile's scales are fetched now and stay in registers through the K loop, so that the epilogue does
    // not start with a dependent round trip to memory: sx (times 1/256, which removes the 16 x 16 of the
    // nibble trick exactly) for the BM tokens, then sw for the BN channels.
    constexpr int NT = 64 * NW;
    constexpr int PRE = (ROWS + NT - 1) / NT;
    float pre[PRE];
    if constexpr (MODE != MODE_I32) {
#pragma unroll
        for (int q = 0; q < PRE; ++q) {
            const int idx = tid + NT * q;
            pre[q] = 0.f;
            // (the asymmetric epilogue removes the factor 256 by a shift before its zero-point correction)
            if (idx < BM) pre[q] = sx[min(m0 + idx, T - 1)] * (MODE == MODE_ASYM ? 1.f : 1.f / 256.f);
            else if (idx < ROWS) pre[q] = sw[min(n0 + idx - BM, N - 1)];
        }
    }
    // asymmetric codes: the tokens' zero points and the channels' weight row sums travel the same way
    int prez[PRE];
    if constexpr (MODE == MODE_ASYM) {
#pragma unroll
        for (int q = 0; q < PRE; ++q) {
            const int idx = tid + NT * q;
            prez[q] = 0;
            if (idx < BM) prez[q] = zx[min(m0 + idx, T - 1)];
            else if (idx < ROWS) prez[q] = wsum[min(n0 + idx - BM, N - 1)];
        }
    }
    // whole: the K step is a full one, every lane takes part (no predicate, hence no control flow)
    // Where the blocks divide evenly among the waves, a wave's first A_SLOTS slots read tokens and the others
    // channels, whatever the wave: the operand of a slot is then known at compile time and the two bases of a K
    // step (kbase) are computed once per step on the scalar unit instead of once per DMA.
    constexpr bool SLOTS_STATIC = (BLKS % NW == 0) && ((BM / RPB) % NW == 0);
    constexpr int A_SLOTS = (BM / RPB) / NW;
    struct KBase { const uint8_t* a; const uint8_t* b; };
    auto kbase = [&](int kt) { return KBase{qx + (int64_t)kt * RB, qw + (int64_t)kt * RB}; };
    auto issue_slot = [&](int stage, const KBase& kbs, int s, auto whole) {
        const int blk = (wave + NW * s) % BLKS;
        const uint8_t* base = (SLOTS_STATIC ? s < A_SLOTS : blk < BM / RPB) ? kbs.a : kbs.b;
        if (decltype(whole)::value || kcl[s] < tail_chunks) dma16(base, voff[s], lds0 + stage * STAGE + blk * 1024);
    };
    auto issue = [&](int stage, int kt) {
        const KBase kbs = kbase(kt);
#pragma unroll
        for (int s = 0; s < CH; ++s) {
            if (kt == KT - 1) issue_slot(stage, kbs, s, std::false_type{});
            else issue_slot(stage, kbs, s, std::true_type{});
        }
    };

    i32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    const int frow = lane & 31, fk = lane >> 5;
    // LDS byte offsets of this lane's fragments within a stage for the wave's first sub-step; sub-step s reads
    // logical chunk 2 s + fk, i.e. position (2 s + fk) ^ swz(r) = (fk ^ swz(r)) ^ 2 s (s_off is 0 or a power
    // of two above the wave's own sub-step bits, so it can be folded in here).
    int aoff[FM], boff[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int r = wm * WM + 32 * i + frow;
        aoff[i] = (r * RB + ((fk ^ swz<RB>(r)) << 4)) ^ (s_off << 5);
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int r = BM + wn * WN + 32 * j + frow;
        boff[j] = (r * RB + ((fk ^ swz<RB>(r)) << 4)) ^ (s_off << 5);
    }
    struct Frags { u32x4 a[FM], b[FN]; };                         // 32 packed codes per lane and fragment
    struct Unpacked { i32x4 alo[FM], ahi[FM], blo[FN], bhi[FN]; };   // the same as int8 x 16 MFMA operands
    auto load_frags = [&](Frags& f, const unsigned char* stage, int s) {
#pragma unroll
        for (int i = 0; i < FM; ++i) f.a[i] = *reinterpret_cast<const u32x4*>(stage + (aoff[i] ^ (s << 5)));
#pragma unroll
        for (int j = 0; j < FN; ++j) f.b[j] = *reinterpret_cast<const u32x4*>(stage + (boff[j] ^ (s << 5)));
    };
    auto unpack = [&](const Frags& f, Unpacked& u) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            u32x4 w = f.a[i];
            // unsigned codes c: c ^ 8 read as a signed nibble is c - 8; the epilogue adds 8 * wsum back
            if (MODE == MODE_ASYM) w ^= 0x88888888u;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                u.alo[i][e] = (int)((w[e] & 0x0F0F0F0Fu) << 4);
                u.ahi[i][e] = (int)(w[e] & 0xF0F0F0F0u);
            }
        }
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                u.blo[j][e] = (int)((f.b[j][e] & 0x0F0F0F0Fu) << 4);
                u.bhi[j][e] = (int)(f.b[j][e] & 0xF0F0F0F0u);
            }
    };
    // The same two steps cut into NPART parts (part c of the fragments' dwords, part c of the matrix
    // instructions), for the region that also issues the DMA of a later K step: one DMA instruction goes
    // between consecutive parts, so that the matrix pipe works through part c while the wave is held up
    // issuing the DMA.
    constexpr int NPART = CH;
    constexpr int NITEM = 4 * (FM + FN);          // dwords to unpack per sub-step
    auto unpack_part = [&](const Frags& f, Unpacked& u, int c) {
#pragma unroll
        for (int q = 0; q < NITEM; ++q) {
            if (q * NPART / NITEM != c) continue;
            const int fr = q >> 2, e = q & 3;
            if (fr < FM) {
                uint32_t w = f.a[fr][e];
                if (MODE == MODE_ASYM) w ^= 0x88888888u;
                u.alo[fr][e] = (int)((w & 0x0F0F0F0Fu) << 4);
                u.ahi[fr][e] = (int)(w & 0xF0F0F0F0u);
            } else {
                const uint32_t w = f.b[fr - FM][e];
                u.blo[fr - FM][e] = (int)((w & 0x0F0F0F0Fu) << 4);
                u.bhi[fr - FM][e] = (int)(w & 0xF0F0F0F0u);
            }
        }
    };
    auto mfma_part = [&](const Unpacked& u, int c) {
#pragma unroll
        for (int m = 0; m < 2 * FM * FN; ++m) {
            if (m * NPART / (2 * FM * FN) != c) continue;
            const int i = m / (2 * FN), j = (m >> 1) % FN;
            if ((m & 1) == 0) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.blo[j], u.alo[i], acc[i][j], 0, 0, 0);
            else acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.bhi[j], u.ahi[i], acc[i][j], 0, 0, 0);
        }
    };
    auto mfma_all = [&](const Unpacked& u) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.blo[j], u.alo[i], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.bhi[j], u.ahi[i], acc[i][j], 0, 0, 0);
            }
    };
    // Scheduling request for one sub-step region (the LDS reads of sub-step g + 2, the unpack arithmetic
    // of g + 1, the matrix instructions of g): reads first, then the unpack instructions spread evenly
    // behind the matrix instructions, where a single wave issues them while the matrix pipe is busy.
    constexpr int NMFMA = 2 * FM * FN;
    constexpr int NVALU = (FM + FN) * 12 + (MODE == MODE_ASYM ? FM * 4 : 0);
    constexpr int VPM = (NVALU + NMFMA - 1) / NMFMA;
    auto interleave = [&](bool with_reads) {
        if (with_reads) __builtin_amdgcn_sched_group_barrier(0x100, FM + FN, 0);
#pragma unroll
        for (int m = 0; m < NMFMA; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);
        }
    };

    // Software pipeline over sub-steps g = kt NSUB + s (K step kt lives in stage kt % NSTAGE):
    //   region g:  read the fragments of g + 2 | unpack those of g + 1 | matrix cores on g.
    // Before the region whose read first touches K step kt + 1 (s = NSUB - 2) every read of K step kt has
    // been issued: wait for the DMA of kt + 1, barrier (now every wave has left the stage of kt), and
    // start the DMA of K step kt + NSTAGE into that stage.  Every K step issues the same number of DMA
    // instructions (beyond the end the last step is loaded again into a stage nobody reads), so the
    // wait count is a constant: the NSTAGE - 2 newest groups may still be in flight.
    if constexpr (!LOADER) {
#pragma unroll
        for (int st = 0; st < NSTAGE; ++st) issue(st, min(st, KT - 1));
        wait_vm<(NSTAGE - 1) * CH>();
    }
    lds_barrier();
    Frags raw[2];
    Unpacked unp[2];
    load_frags(raw[0], smem, 0);
    load_frags(raw[1], smem, 1);
    unpack(raw[0], unp[0]);
    int cur = 0;                    // stage of K step kt
    // One K step kt living in stage curc (an int, or an integral constant: then every LDS address of the step is a
    // register plus an immediate); whole: the K step whose DMA it issues is a full one.
    auto k_step = [&](int kt, auto curc, auto whole) {
        const int cs = curc;
        const int nxt = (cs == NSTAGE - 1) ? 0 : cs + 1;
        const unsigned char* scur = smem + cs * STAGE;
        const unsigned char* snxt = smem + nxt * STAGE;
#pragma unroll
        for (int s = 0; s < NSUB; ++s) {
            if (s == NSUB - 2) {
                if constexpr (!LOADER) wait_vm<(NSTAGE - 2) * CH>();
                lds_barrier();      // stage nxt has landed for every wave; every wave has left stage cur
            }
            if (s + 2 < NSUB) load_frags(raw[s & 1], scur, s + 2);
            else load_frags(raw[s & 1], snxt, s + 2 - NSUB);
            if (LOADER || s != NSUB - 2) {
                unpack(raw[(s + 1) & 1], unp[(s + 1) & 1]);
                mfma_all(unp[s & 1]);
                interleave(true);
            } else {
                // the region after the barrier also refills stage cur with K step kt + NSTAGE, one DMA
                // instruction after each part of the matrix work
                const KBase kbs = kbase(min(kt + NSTAGE, KT - 1));
#pragma unroll
                for (int c = 0; c < NPART; ++c) {
                    unpack_part(raw[(s + 1) & 1], unp[(s + 1) & 1], c);
                    mfma_part(unp[s & 1], c);
                    if (c == 0) __builtin_amdgcn_sched_group_barrier(0x100, FM + FN, 0);
                    constexpr int MPP = (NMFMA + NPART - 1) / NPART;       // most matrix instructions of a part
#pragma unroll
                    for (int m = 0; m < MPP; ++m) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    issue_slot(cs, kbs, c, whole);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };
    // K steps [k0, k1) starting in stage `cur`
    auto k_steps = [&](int k0, int k1, auto whole) {
        for (int kt = k0; kt < k1; ++kt) {
            k_step(kt, cur, whole);
            cur = (cur == NSTAGE - 1) ? 0 : cur + 1;
        }
    };
    // The steps that fetch the shortened last K step (a lane predicate, hence control flow between the
    // matrix instructions) are kept apart from the bulk, whose DMA is unconditional.
    const int k_whole = (tail_chunks == CPR) ? KT - 1 : max(0, KT - 1 - NSTAGE);
    // the bulk in rounds of NSTAGE steps, so that each step's stage is a compile-time constant
    int kt0 = 0;
    for (; kt0 + NSTAGE <= k_whole; kt0 += NSTAGE)
        static_for<NSTAGE>([&](auto c) { k_step(kt0 + c, c, std::true_type{}); });
    k_steps(kt0, k_whole, std::true_type{});
    k_steps(k_whole, KT - 1, std::false_type{});
    {
        const unsigned char* scur = smem + cur * STAGE;
#pragma unroll
        for (int s = 0; s < NSUB; ++s) {
            if (s_off + s < tail_sub) {                      // wave-uniform
                if (s + 2 < NSUB && s_off + s + 2 < tail_sub) load_frags(raw[s & 1], scur, s + 2);
                if (s + 1 < NSUB && s_off + s + 1 < tail_sub) unpack(raw[(s + 1) & 1], unp[(s + 1) & 1]);
                mfma_all(unp[s & 1]);
            }
        }
    }
    if constexpr (!LOADER) wait_vm<0>();
    lds_barrier();

    // ---- K split: wave kh finishes the token blocks i of half kh; it hands the other half's partial sums to
    // its partner (same wave tile, other K half) through LDS and adds the partner's to its own.
    if constexpr (KS == 2) {
        constexpr int HF = FM / 2;
        int* give = reinterpret_cast<int*>(smem + (size_t)wave * XCH);
        const int* take = reinterpret_cast<const int*>(smem + (size_t)(wave ^ (WGM * WGN)) * XCH);
        static_assert(((WGM * WGN) & (WGM * WGN - 1)) == 0, "the partner is the wave with the other kh bit");
        auto hand_over = [&](auto khc) {
            constexpr int OTHER = (1 - decltype(khc)::value) * HF;
#pragma unroll
            for (int ii = 0; ii < HF; ++ii)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) give[((ii * FN + j) * 16 + e) * 64 + lane] = acc[OTHER + ii][j][e];
        };
        auto add_partner = [&](auto khc) {
            constexpr int MINE = decltype(khc)::value * HF;
#pragma unroll
            for (int ii = 0; ii < HF; ++ii)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[MINE + ii][j][e] += take[((ii * FN + j) * 16 + e) * 64 + lane];
        };
        if (kh == 0) hand_over(std::integral_constant<int, 0>{});
        else hand_over(std::integral_constant<int, 1>{});
        lds_barrier();
        if (kh == 0) add_partner(std::integral_constant<int, 0>{});
        else add_partner(std::integral_constant<int, 1>{});
        lds_barrier();                                      // the stages are reused below
    }

    // The token blocks i this wave finishes: all FM of its tile, or with a K split the half kh.
    constexpr int IH = FM / KS;
    auto epilogue = [&](auto khc) {
        constexpr int I0 = decltype(khc)::value * IH;
        // ---- epilogue.  Accumulator element e of block (i, j): output channel
        // n0 + wn WN + 32 j + 8 (e / 4) + 4 fk + e % 4, token m0 + wm WM + 32 i + frow.
        if constexpr (MODE == MODE_I32) {
    #pragma unroll
            for (int ii = 0; ii < IH; ++ii) {
                const int i = I0 + ii;
                const int t = m0 + wm * WM + 32 * i + frow;
    #pragma unroll
                for (int j = 0; j < FN; ++j)
    #pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int n = n0 + wn * WN + 32 * j + 8 * (e >> 2) + 4 * fk + (e & 3);
                        if (t < T && n < N) static_cast<int32_t*>(out)[(int64_t)t * ldo + n] = acc[i][j][e] >> 8;
                    }
            }
        } else {
            // all waves are past the last barrier of the K loop: the stages are free for staging
            unsigned char* slab = smem + (size_t)wave * SLAB;
            float* sc = reinterpret_cast<float*>(smem + (size_t)NW * SLAB);     // [BM] token scales, [BN] channel scales
            int* zc = reinterpret_cast<int*>(sc + ROWS);                        // [BM] zero points, [BN] weight row sums
    #pragma unroll
            for (int q = 0; q < PRE; ++q) {
                const int idx = tid + NT * q;
                if (idx < ROWS) {
                    sc[idx] = pre[q];
                    if constexpr (MODE == MODE_ASYM) zc[idx] = prez[q];
                }
            }
            lds_barrier();
            f32x4 swv[FN][4];
            int wsv[FN][4][4];
    #pragma unroll
            for (int j = 0; j < FN; ++j)
    #pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    swv[j][eg] = *reinterpret_cast<const f32x4*>(sc + BM + wn * WN + 32 * j + 8 * eg + 4 * fk);
                    if (MODE == MODE_ASYM) {
    #pragma unroll
                        for (int q = 0; q < 4; ++q) wsv[j][eg][q] = zc[BM + wn * WN + 32 * j + 8 * eg + 4 * fk + q];
                    }
                }
            uint16_t* y = static_cast<uint16_t*>(out);
    #pragma unroll
            for (int ii = 0; ii < IH; ++ii) {
                const int i = I0 + ii;
                const int t = min(m0 + wm * WM + 32 * i + frow, T - 1);
                const float sxs = sc[wm * WM + 32 * i + frow];
                int zoff = 0;
                if (MODE == MODE_ASYM) zoff = zc[wm * WM + 32 * i + frow] - 8;
    #pragma unroll
                for (int j = 0; j < FN; ++j)
    #pragma unroll
                    for (int eg = 0; eg < 4; ++eg) {
                        float f[4];
    #pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            int a = acc[i][j][4 * eg + q];
                            // sum (c - 8) w - (z - 8) wsum = sum (c - z) w, at most 120 d_e in magnitude: formed
                            // after the exact shift, so that it is not held to the x256 range
                            if (MODE == MODE_ASYM) a = (a >> 8) - zoff * wsv[j][eg][q];
                            f[q] = (float)a * sxs * swv[j][eg][q];
                        }
                        const u32x2 pk = u32x2{pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3])};
                        *reinterpret_cast<u32x2*>(slab + frow * (WN * 2) + (32 * j + 8 * eg + 4 * fk) * 2) = pk;
                    }
                // the slab is private to the wave: no workgroup barrier, only this wave's LDS traffic
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                const int tbase = m0 + wm * WM + 32 * i, nbase = n0 + wn * WN;
                if (vec_store) {
                    constexpr int CPS = WN / 8;                   // 16-byte chunks per slab row
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
                            y[(int64_t)(tbase + row) * ldo + nbase + col] =
                                *reinterpret_cast<const uint16_t*>(slab + row * (WN * 2) + col * 2);
                    }
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
        }
    };
    if (KS == 1 || kh == 0) epilogue(std::integral_constant<int, 0>{});
    else epilogue(std::integral_constant<int, KS - 1>{});
}

// The kernel instantiation's name as a profiler prints it (template arguments in order), per output mode.
template <int BM, int BN, int WGM, int WGN, int RB, int NSTAGE, int KS, bool LOADER>
const char* tile_name(int mode) {
    auto make = [](int m) {
        char buf[96];
        snprintf(buf, sizeof buf, "k_gemm_mfma<%d, %d, %d, %d, %d, %d, %d, %d, %s>", BM, BN, WGM, WGN, RB, NSTAGE, m, KS,
                 LOADER ? "true" : "false");
        return std::string(buf);
    };
    static const std::string names[3] = {make(MODE_BF16), make(MODE_ASYM), make(MODE_I32)};
    return names[mode].c_str();
}

template <int BM, int BN, int WGM, int WGN, int RB, int NSTAGE, int KS = 1, bool LOADER = false>
pme_status launch_tile(const GemmArgs& a) {
    const int kb = (int)(a.d_e / 2);
    if (kb % 64) return PME_ERR_UNSUPPORTED_PATH;      // whole sub-steps; the last K step may be half as long
    if ((int64_t)std::max(a.T, a.N) * kb >= (int64_t(1) << 32)) return PME_ERR_UNSUPPORTED_PATH;   // 32-bit DMA offsets
    if (a.dry) {
        if (a.plan) *a.plan = tile_name<BM, BN, WGM, WGN, RB, NSTAGE, KS, LOADER>(a.out_i32 ? MODE_I32 : a.zx ? MODE_ASYM : MODE_BF16);
        return PME_OK;
    }
    const int tiles_m = (int)((a.T + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(64 * (WGM * WGN * KS + (LOADER ? 1 : 0)));
    const size_t lds = (size_t)NSTAGE * (BM + BN) * RB;
    if (lds > 64 * 1024) {
        static std::atomic<uint32_t> done[3];
        if (allow_dynamic_lds(k_gemm_mfma<BM, BN, WGM, WGN, RB, NSTAGE, MODE_BF16, KS, LOADER>, (int)lds, done[0]) != PME_OK ||
            allow_dynamic_lds(k_gemm_mfma<BM, BN, WGM, WGN, RB, NSTAGE, MODE_ASYM, KS, LOADER>, (int)lds, done[1]) != PME_OK ||
            allow_dynamic_lds(k_gemm_mfma<BM, BN, WGM, WGN, RB, NSTAGE, MODE_I32, KS, LOADER>, (int)lds, done[2]) != PME_OK)
            return PME_ERR_HIP;
    }
    // 16-byte output pieces need 8-element alignment of N, the pitch and the base
    const int vec = (a.N % 8 == 0 && a.ldy % 8 == 0 && (reinterpret_cast<uintptr_t>(a.y) & 15) == 0) ? 1 : 0;
#define PME_LAUNCH(MODE)                                                                                        \
    hipLaunchKernelGGL((k_gemm_mfma<BM, BN, WGM, WGN, RB, NSTAGE, MODE, KS, LOADER>), grid, block, lds, a.stream, a.qx, a.qw, \
                       a.sx, a.sw, a.zx, a.wsum, (int)a.T, (int)a.N, kb, a.y, a.ldy, tiles_m, tiles_n, xcd_grid_m(tiles_m, tiles_n, BM, BN), vec)
    if (a.out_i32) PME_LAUNCH(MODE_I32);
    else if (a.zx) PME_LAUNCH(MODE_ASYM);
    else PME_LAUNCH(MODE_BF16);
#undef PME_LAUNCH
    return hip_status(hipGetLastError());
}

int g_tile_override = 0;

}  // namespace

void set_gemm_tile_override(int id) { g_tile_override = id; }

pme_status launch_gemm_mfma(const GemmArgs& a) {
    // d_e a multiple of 128 (whole K steps), 16-byte aligned rows, and the x256 accumulator in range:
    // 256 * 64 * d_e < 2^31 needs d_e < 2^17.
    if (a.d_e % 128 || a.d_e >= (1 << 17)) return PME_ERR_UNSUPPORTED_PATH;   // tiles with 128-byte rows need d_e % 256 == 0
    if ((reinterpret_cast<uintptr_t>(a.qx) & 15) || (reinterpret_cast<uintptr_t>(a.qw) & 15)) return PME_ERR_UNSUPPORTED_PATH;
    if (a.zx && a.out_i32) return PME_ERR_UNSUPPORTED_PATH;
    const int64_t cus = 256;
    auto tiles = [&](int bm, int bn) { return ((a.T + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
    int id = g_tile_override;
    if (id == 0) {
        // The largest tile that still gives every one of the 256 compute units a workgroup, with whole
        // 128-byte lines per row and K step (measured faster on MI355X than 64-byte steps).
        // (a half-length last step is supported but measured no faster than 64-byte steps, so those are kept
        // when d_e is not a multiple of 256)
        const bool wide = (a.d_e % 256) == 0;
        // (with 64-byte steps 128 x 192 on 4 waves beats 128 x 256 on 8 by a quarter; a fifth wave that does the
        // DMA gains another 3-4 % there, and 1-2 % at 128 x 128 over splitting K between wave pairs)
        if (tiles(128, 128) >= cus * 3 / 4) {
            // Large outputs: the cheapest of four tile shapes by rounds x tile area / efficiency.  The efficiencies
            // are each shape's measured rate on outputs of many rounds, relative to 256 x 256; a round is one
            // workgroup on every compute unit, except that two 128 x 192 workgroups without loader wave share a
            // unit (a pair takes about 1.7 x one, and a unit with a second workgroup about 1.5 x).  The model
            // ranks the shapes as 14 measured outputs from 512 x 14336 to 4096 x 4096 do.
            auto rounds = [&](int64_t t) { return (double)((t + cus - 1) / cus); };
            auto rounds_shared = [&](int64_t t) {
                const int64_t pairs = (t - 1) / (2 * cus);
                const double rest = (double)(t - 2 * cus * pairs) / (double)cus;       // (0, 2]
                return 1.7 * (double)pairs + (rest <= 1.0 ? 1.0 : 1.5 + 0.2 * (rest - 1.0));
            };
            const double c256 = rounds(tiles(256, 256)) * (256.0 * 256.0) / 1.00;
            const double c16 = rounds(tiles(128, 256)) * (128.0 * 256.0) / 0.87;
            const double c192 = rounds_shared(tiles(128, 192)) * (128.0 * 192.0) / 0.83;
            const double c128 = rounds(tiles(128, 128)) * (128.0 * 128.0) / 0.76;
            const double best = std::min(std::min(c256, c16), std::min(c192, c128));
            if (best == c256) id = wide ? 11 : 8;
            else if (best == c16) id = wide ? 16 : 2;
            else if (best == c192) id = tiles(128, 192) <= cus ? (wide ? 28 : 21) : 9;     // the loader's registers allow one workgroup per unit
            else id = wide ? 25 : 22;   // whole 128-byte lines per K step halve the barriers of the loader tile: 3-4 % at 2048 x 2048 x 8704
        }
        // smaller outputs (measured on 18 shapes from 96 to 1536 tokens): 64 x 64, which beats 64 x 128 until the
        // latter has one and a half tiles per compute unit
        // (with whole 128-byte lines per K step -- half the barriers -- where d_e allows: 64 x 64 another 5-13 % on four
        // such shapes, 64 x 128 2-3 %)
        else if (tiles(64, 128) >= cus * 3 / 2) id = wide ? 26 : 23;
        else id = wide ? 27 : 24;
    }
    switch (id) {
        case 1: return launch_tile<256, 256, 2, 4, 64, 3>(a);      // 8 waves of 128 x 64
        case 2: return launch_tile<128, 256, 2, 4, 64, 3>(a);      // 8 waves of 64 x 64
        case 3: return launch_tile<128, 192, 4, 2, 64, 3>(a);      // 8 waves of 32 x 96
        case 4: return launch_tile<128, 128, 2, 4, 64, 3>(a);      // 8 waves of 64 x 32
        case 5: return launch_tile<128, 128, 2, 2, 64, 3>(a);      // 4 waves of 64 x 64
        case 6: return launch_tile<64, 128, 2, 2, 64, 3>(a);       // 4 waves of 32 x 64
        case 7: return launch_tile<64, 64, 2, 2, 64, 3>(a);        // 4 waves of 32 x 32
        case 8: return launch_tile<256, 256, 2, 2, 64, 3>(a);      // 4 waves of 128 x 128
        case 9: return launch_tile<128, 192, 2, 2, 64, 3>(a);      // 4 waves of 64 x 96
        case 10: return launch_tile<256, 128, 4, 2, 64, 3>(a);     // 8 waves of 64 x 64
        // whole 128-byte lines per row and K step
        case 11: return launch_tile<256, 256, 2, 2, 128, 2>(a);    // 4 waves of 128 x 128
        case 12: return launch_tile<256, 256, 2, 4, 128, 2>(a);    // 8 waves of 128 x 64
        case 13: return launch_tile<128, 128, 2, 2, 128, 3>(a);    // 4 waves of 64 x 64
        case 14: return launch_tile<128, 128, 2, 4, 128, 3>(a);    // 8 waves of 64 x 32
        case 15: return launch_tile<128, 192, 2, 2, 128, 3>(a);    // 4 waves of 64 x 96
        case 16: return launch_tile<128, 256, 2, 4, 128, 3>(a);    // 8 waves of 64 x 64
        case 17: return launch_tile<256, 128, 4, 2, 128, 3>(a);    // 8 waves of 64 x 64
        case 18: return launch_tile<256, 128, 2, 2, 128, 3>(a);    // 4 waves of 128 x 64
        // two waves per wave tile, each taking half of every K step
        case 19: return launch_tile<128, 128, 1, 2, 128, 3, 2>(a); // 2 x 2 waves of 128 x 64
        case 20: return launch_tile<128, 192, 1, 2, 128, 3, 2>(a); // 2 x 2 waves of 128 x 96
        // a fifth wave issues all the DMA
        case 21: return launch_tile<128, 192, 2, 2, 64, 3, 1, true>(a);    // 4 waves of 64 x 96 + loader
        case 22: return launch_tile<128, 128, 2, 2, 64, 3, 1, true>(a);    // 4 waves of 64 x 64 + loader
        case 23: return launch_tile<64, 128, 2, 2, 64, 3, 1, true>(a);     // 4 waves of 32 x 64 + loader
        case 24: return launch_tile<64, 64, 2, 2, 64, 3, 1, true>(a);      // 4 waves of 32 x 32 + loader
        case 25: return launch_tile<128, 128, 2, 2, 128, 3, 1, true>(a);   // 4 waves of 64 x 64 + loader, 128-byte rows
        case 26: return launch_tile<64, 128, 2, 2, 128, 3, 1, true>(a);    // 4 waves of 32 x 64 + loader, 128-byte rows
        case 27: return launch_tile<64, 64, 2, 2, 128, 3, 1, true>(a);     // 4 waves of 32 x 32 + loader, 128-byte rows
        case 28: return launch_tile<128, 192, 2, 2, 128, 3, 1, true>(a);   // 4 waves of 64 x 96 + loader, 128-byte rows
    }
    return PME_ERR_UNSUPPORTED_PATH;
}

}  // namespace pme
