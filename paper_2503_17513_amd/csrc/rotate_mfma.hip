// Rotate + quantize on the matrix cores: one workgroup per token (one wave per token where a token is a
// single wave's work, see MULTI below).
//
// Per token (paper Section 3, X_hat = X H_hat, H = P_b (x) S_{2^k}, index i = a 2^k + c):
//   1. the token's d inputs are loaded once, coalesced, and laid out in LDS as bf16 MFMA
//      operand fragments of X~^T (rows c, contraction index a);
//   2. base block: Z^T[c][a'] = sum_a X~[a][c] P[a][a'] with v_mfma_f32_16x16x32_bf16.  The +-1
//      entries of P are exact in bf16, bf16 inputs are exact, fp32 inputs are split into three
//      bf16 terms whose sum is exact, so every product is exact and accumulation is fp32.
//      Only the ceil(d / 2^k) base rows that hold real inputs enter the contraction: the
//      zero padding of the expansion is never read or materialised;
//   3. FWHT along c in registers.  A lane owns one a' and 4 * (2^k / 16) values of c; two of
//      the k butterfly stages live on lane bits 4 and 5 and are turned into register stages
//      by v_permlane16_swap / v_permlane32_swap, which also leaves every lane with a
//      contiguous run of 2^(k-2) outputs;
//   4. per-token absmax (or min/max) by wavefront reduction, combined across waves in LDS;
//   5. codes by one fused multiply-add with a rounding constant (round half to even),
//      packed eight to a dword and stored in runs of 2^(k-3) bytes per lane.
// Waves split the token by a' (16-wide tiles, TPW tiles per wave); the FWHT never crosses a'.
// Since S_{2^k} = S_{2^f} (x) S_{2^(k-f)}, the launcher may hand the kernel the same H as a larger block
// P_b (x) S_{2^f} times fewer columns (see launch_rotate_mfma): steps 2 and 3 are unaware of it.
#include "pme_internal.h"

#include <algorithm>
#include <mutex>
#include <type_traits>
#include <vector>

namespace pme {
namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kMaxWaves = 10;   // waves per workgroup: 10 column tiles of 16 (order 160) at one tile per wave

template <int KLOG2> struct Layout {
    static constexpr int NC = 1 << KLOG2;      // FWHT length
    static constexpr int MT = NC / 16;         // 16-row MFMA tiles along c
    static constexpr int NREG = MT * 4;        // values per lane per a'-tile
    static constexpr int NBITS = KLOG2 - 2;    // register index bits
    static constexpr int RUN = NC / 4;         // contiguous outputs per lane after the FWHT
    // Position (within the lane's contiguous run) of register index idx after the FWHT.
    // Before: idx bit 0,1 = c0,c1; idx bits 2.. = c4..c(k-1); lane bit 4 = c2, lane bit 5 = c3.
    // After (k >= 6): the two top idx bits hold c2, c3; lane bits 4, 5 hold c(k-2), c(k-1).
    // After (k == 5): idx bits = c0, c1, c2; lane bit 4 = c4, lane bit 5 = c3.
    static constexpr int run_pos(int idx) {
        if (KLOG2 == 5) return idx;
        int lo = idx & 3;
        int mid = (idx >> 2) & ((1 << (NBITS - 4)) - 1);     // c4 .. c(k-3)
        int c2 = (idx >> (NBITS - 2)) & 1, c3 = (idx >> (NBITS - 1)) & 1;
        return lo | (c2 << 2) | (c3 << 3) | (mid << 4);
    }
    // inverse of run_pos as a constant table, so that an unrolled loop indexes registers with constants
    struct Table { int v[NC / 4]; };
    static constexpr Table make_table() {
        Table t{};
        for (int idx = 0; idx < NREG; ++idx) t.v[run_pos(idx)] = idx;
        return t;
    }
    static constexpr Table kRegOfRun = make_table();
    static constexpr int reg_of_run_pos(int j) { return kRegOfRun.v[j]; }
};

__device__ __forceinline__ void swap16(float& r0, float& r1) {
    // lane bit 4 <-> the register bit that distinguishes r0 / r1
    u32x2 v = __builtin_amdgcn_permlane16_swap(__float_as_uint(r0), __float_as_uint(r1), false, false);
    r0 = __uint_as_float(v.x);
    r1 = __uint_as_float(v.y);
}
__device__ __forceinline__ void swap32(float& r0, float& r1) {
    u32x2 v = __builtin_amdgcn_permlane32_swap(__float_as_uint(r0), __float_as_uint(r1), false, false);
    r0 = __uint_as_float(v.x);
    r1 = __uint_as_float(v.y);
}

template <int NREG, int BIT> __device__ __forceinline__ void butterfly(float (&v)[NREG]) {
#pragma unroll
    for (int i = 0; i < NREG; ++i)
        if (!(i & (1 << BIT))) {
            const float u = v[i], w = v[i | (1 << BIT)];
            v[i] = u + w;
            v[i | (1 << BIT)] = u - w;
        }
}
template <int NREG, int BIT> __device__ __forceinline__ void lane_swap16(float (&v)[NREG]) {
#pragma unroll
    for (int i = 0; i < NREG; ++i)
        if (!(i & (1 << BIT))) swap16(v[i], v[i | (1 << BIT)]);
}
template <int NREG, int BIT> __device__ __forceinline__ void lane_swap32(float (&v)[NREG]) {
#pragma unroll
    for (int i = 0; i < NREG; ++i)
        if (!(i & (1 << BIT))) swap32(v[i], v[i | (1 << BIT)]);
}

template <int NREG, int BIT> struct RegStages {
    static __device__ __forceinline__ void run(float (&v)[NREG]) {
        butterfly<NREG, BIT>(v);
        RegStages<NREG, BIT - 1>::run(v);
    }
};
template <int NREG> struct RegStages<NREG, -1> {
    static __device__ __forceinline__ void run(float (&)[NREG]) {}
};

template <int KLOG2> __device__ __forceinline__ void fwht_lane(float (&v)[Layout<KLOG2>::NREG]) {
    using L = Layout<KLOG2>;
    RegStages<L::NREG, L::NBITS - 1>::run(v);          // every c bit that starts in a register
    if constexpr (KLOG2 == 5) {
        lane_swap16<L::NREG, 2>(v);                    // idx bit 2: c4 -> c2
        butterfly<L::NREG, 2>(v);
        lane_swap32<L::NREG, 2>(v);                    // idx bit 2: c2 -> c3 (lane bit 5 now c2)
        butterfly<L::NREG, 2>(v);
        lane_swap32<L::NREG, 2>(v);                    // back: idx bit 2 = c2, lane bit 5 = c3
    } else {
        lane_swap16<L::NREG, L::NBITS - 2>(v);
        lane_swap32<L::NREG, L::NBITS - 1>(v);
        butterfly<L::NREG, L::NBITS - 2>(v);
        butterfly<L::NREG, L::NBITS - 1>(v);
    }
}

// First output column of this lane's run, for lane bits (l4, l5).
template <int KLOG2> __device__ __forceinline__ int run_start(int l4, int l5) {
    using L = Layout<KLOG2>;
    if (KLOG2 == 5) return 8 * l5 + 16 * l4;
    return L::RUN * (l4 + 2 * l5);
}

__device__ __forceinline__ float wave_max(float v) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}
__device__ __forceinline__ float wave_min(float v) {
    for (int off = 32; off > 0; off >>= 1) v = fminf(v, __shfl_xor(v, off));
    return v;
}

// bf16 bits of the truncation of f, and the exact remainder.
__device__ __forceinline__ uint32_t split_hi(float f, float& rem) {
    const uint32_t hi = __float_as_uint(f) & 0xFFFF0000u;
    rem = f - __uint_as_float(hi);
    return hi >> 16;
}

// ---------------------------------------------------------------------------------------------
// B-operand table: the Paley block as ready-made bf16 MFMA fragments, built once per
// (device, b, folded stages, real base rows) by a small kernel and kept in device memory owned by the library.
// Entry (tile, ks), lane (a' = 16 tile + lane % 16, g = lane / 16) holds P[32 ks + 8 g + e][a'],
// e = 0..7 (+-1 in bf16; 0 outside the block or beyond the rows that hold real inputs).
// ---------------------------------------------------------------------------------------------
constexpr int kMaxTiles = 22, kMaxKs = 7;     // blocks up to order 352, up to 224 real base rows
constexpr int kPoolEntries = 16384;           // 16 MB of fragments per device: a shape takes 7 to 154 KB of it
typedef u32x4 Fragment[64];                   // one 16 x 32 B-operand tile: 16 bytes per lane
__device__ __align__(256) Fragment g_fragment_pool[kPoolEntries];

// Fragments of the base block B = P_b (x) S_{2^fold} of order b 2^fold (fold = 0: the Paley block itself).
// Folding the first `fold` butterfly stages into the block leaves H = P_b (x) S_{2^k} unchanged, since
// S_{2^k} = S_{2^fold} (x) S_{2^(k - fold)}: entry ((a, u), (a', u')) = P[a][a'] (-1)^popcount(u & u').
// One workgroup per (tile, ks); table[tile * kMaxKs + ks] is the fragment.
__global__ void __launch_bounds__(64) k_fill_ptable(Fragment* table, int b, int fold, int rows) {
    __shared__ signed char chi[512];
    const int lane = threadIdx.x, q = b - 1, border = b << fold, umask = (1 << fold) - 1;
    if (b > 1) fill_quadratic_character(chi, q, lane, 64);
    const int tile = blockIdx.x / kMaxKs, ks = blockIdx.x % kMaxKs;
    const int ap = tile * 16 + (lane & 15), g = lane >> 4;
    u32x4 pk;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        uint32_t word = 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int a = 32 * ks + 8 * g + 2 * p + h;
            uint32_t bits = 0;
            if (a < rows && a < border && ap < border) {
                int sgn = (b > 1) ? paley_entry(chi, q, a >> fold, ap >> fold) : 1;
                if (__popc((unsigned)(a & ap & umask)) & 1) sgn = -sgn;
                bits = sgn > 0 ? 0x3F80u : 0xBF80u;
            }
            word |= bits << (16 * h);
        }
        pk[p] = word;
    }
    table[blockIdx.x][lane] = pk;
}

struct TableKey { int b, fold, rows; Fragment* table; };
struct DeviceTables {
    Fragment* pool = nullptr;          // this device's copy of g_fragment_pool
    int used = 0;                      // entries handed out
    std::vector<TableKey> keys;
};
constexpr int kMaxDevices = 16;
std::mutex g_table_mutex;
DeviceTables g_tables[kMaxDevices];

// Returns the fragment table for (b, fold, rows) on the current device, building it on a miss: ceil(order / 16)
// tiles of kMaxKs fragments from the device's pool.  A miss launches the fill kernel on `stream` and waits for
// it once, so that callers on other streams never see a half-written table.  Tables are never moved or
// reused: kernels in flight, and HIP graphs that captured a launch, keep reading them.  When the pool is
// used up (hundreds of distinct shapes in one process) a further shape gets PME_ERR_UNSUPPORTED_PATH and the
// automatic path takes the generic kernel for it.
const Fragment* fragment_table(int b, int fold, int rows, hipStream_t stream, pme_status* st) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { *st = PME_ERR_HIP; return nullptr; }
    std::lock_guard<std::mutex> lock(g_table_mutex);
    DeviceTables& D = g_tables[dev];
    for (const TableKey& e : D.keys)
        if (e.b == b && e.fold == fold && e.rows == rows) return e.table;
    if (!D.pool && hipGetSymbolAddress(reinterpret_cast<void**>(&D.pool), HIP_SYMBOL(g_fragment_pool)) != hipSuccess) {
        D.pool = nullptr;
        *st = PME_ERR_HIP;
        return nullptr;
    }
    const int tiles = ((b << fold) + 15) / 16, entries = tiles * kMaxKs;
    if (D.used + entries > kPoolEntries) { *st = PME_ERR_UNSUPPORTED_PATH; return nullptr; }
    // The fill below is waited for, which is not allowed on a stream that is being captured into a graph (it would
    // break the capture): refuse, leaving the capture intact.
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capturing) != hipSuccess) { *st = PME_ERR_HIP; return nullptr; }
    if (capturing != hipStreamCaptureStatusNone) { *st = PME_ERR_COLD_SHAPE; return nullptr; }
    Fragment* table = D.pool + D.used;
    hipLaunchKernelGGL(k_fill_ptable, dim3(entries), dim3(64), 0, stream, table, b, fold, rows);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(stream) != hipSuccess) { *st = PME_ERR_HIP; return nullptr; }
    D.used += entries;
    D.keys.push_back(TableKey{b, fold, rows, table});
    return table;
}

#define PME_AS1 __attribute__((address_space(1)))
#define PME_AS3 __attribute__((address_space(3)))
typedef __attribute__((ext_vector_type(4))) short s16x4;

// Physical LDS position (in 16-byte chunks) of the 8 inputs (a, c .. c+7), c a multiple of 8, in the
// bf16 layout: blocks of 4 rows x 16 columns stored contiguously (128 bytes), so that the 16 lanes of
// a transposing LDS read touch one contiguous 128-byte block.
template <int MT> __device__ __forceinline__ int chunk_of(int a, int c) {
    return ((a >> 2) * MT + (c >> 4)) * 8 + (a & 3) * 2 + ((c >> 3) & 1);
}

// LDS-only barrier and DMA helpers.  The DMA and the waits on it are inline assembly so that the
// compiler does not order LDS reads of the B fragments or of the reduction scratch after them.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void wait_all_vm() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// 16 bytes per lane from global memory into LDS at lds_base + 16 * lane (lds_base wave-uniform); lanes
// switched off by the caller's branch move nothing.  Overwrites M0, which the compiler does not keep
// values in; no other code in this kernel makes the compiler emit an M0 use.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
    // wave-uniform 64-bit base in SGPRs plus a 32-bit byte offset per lane
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}

// One workgroup handles tokens blockIdx.x, blockIdx.x + gridDim.x, ...  The token buffer in LDS is
// refilled for the next token as soon as the matrix-core phase of the current one has consumed it,
// so the HBM read of token i + 1 runs under the FWHT / quantize / store phase of token i.
// Most waves a workgroup of this instantiation is launched with (bounds the registers per lane).
template <int KLOG2, int TPW> constexpr int max_waves() {
    return ((TPW == 1 && KLOG2 <= 8) || KLOG2 == 6) ? kMaxWaves : kMaxWaves / 2;
}

enum { OUT_SYM = 0, OUT_ASYM = 1, OUT_XHAT = 2, OUT_MXFP4 = 3 };   // int4 symmetric / asymmetric codes, fp32 values, MXFP4

// MULTI: a token fits one wave (all its tiles are this wave's TPW tiles), and every wave of the workgroup
// rotates tokens of its own, in a token buffer of its own; only the B fragments are shared.  Compared
// with one-wave workgroups this loads the fragments once per several tokens and hands the dispatcher
// fewer workgroups, which is what counts at small 2^k, where a token is only a few KB.
// BGLOBAL: the P fragments are not staged in LDS but read from the table in device memory (L2) for every
// token: for blocks whose fragments do not fit beside the token buffer (order 312: 140 KB of fragments).
// KSREG > 0 (with BGLOBAL): the workgroup reads its fragments (at most KSREG K steps) once, before the token
// loop, and keeps them in registers.
template <int KLOG2, int TPW, bool F32IN, int OUT, bool MULTI = false, bool BGLOBAL = false, int KSREG = 0>
__global__ void __launch_bounds__((64 * max_waves<KLOG2, TPW>()))
k_rotate_mfma(const void* __restrict__ xv, int64_t ldx, int T, int d, int d_e, int b, int ks_count, const Fragment* __restrict__ ptable,
              double gamma, uint8_t* __restrict__ qx, float* __restrict__ sx, int32_t* __restrict__ zx,
              uint8_t* __restrict__ ex, float* __restrict__ xhat) {
    using L = Layout<KLOG2>;
    constexpr int NC = L::NC, MT = L::MT, NREG = L::NREG;
    constexpr int NS = F32IN ? 3 : 1;
    const int plane_bytes = ks_count * MT * 1024;     // one bf16 copy of the K-padded token

    extern __shared__ __align__(1024) unsigned char smem[];   // NS token planes, then the B fragments
    __shared__ float red[2 * kMaxWaves];

    static_assert(!(MULTI && F32IN), "the multi-token variant takes bf16 input");
    const int lane = threadIdx.x & 63, wave_hw = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nwaves_hw = blockDim.x >> 6;
    // the waves that share a token, and this thread's place among them
    const int wave = MULTI ? 0 : wave_hw, nwaves = MULTI ? 1 : nwaves_hw;
    const int tid = MULTI ? lane : (int)threadIdx.x, nthreads = MULTI ? 64 : (int)blockDim.x;
    const int last_tile = (b + 15) / 16 - 1;          // surplus tile slots of the last wave re-read it
    const int l15 = lane & 15, g = lane >> 4;
    const int rows_k = 32 * ks_count;                 // rows of the K-padded operand
    unsigned char* tsm = smem + (MULTI ? (size_t)wave_hw * NS * plane_bytes : 0);          // this token's planes
    // B fragments: this wave's tiles; MULTI: all tiles, shared by the workgroup's waves
    unsigned char* bsm = smem + (size_t)(MULTI ? nwaves_hw : 1) * NS * plane_bytes + (size_t)wave * TPW * ks_count * 1024;

    const int real_groups = (((d + NC - 1) >> KLOG2) + 3) >> 2;        // 4-row groups holding real inputs
    const int nchunks = real_groups * MT * 8;
    if constexpr (!F32IN) {
        // chunks of the K-padded operand that hold no input are zero and are never written again
        const int first = ((d >> KLOG2) >> 2) * MT * 8;
        const int total = (rows_k >> 2) * MT * 8;
        for (int p = first + tid; p < total; p += nthreads) {
            const int blk = p >> 3, r = p & 7;
            const int a = 4 * (blk / MT) + (r >> 1), c = 16 * (blk % MT) + 8 * (r & 1);
            if (a * NC + c >= d) *reinterpret_cast<u32x4*>(tsm + (size_t)p * 16) = u32x4{0u, 0u, 0u, 0u};
        }
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(PME_AS3 unsigned char*)tsm;

    // bf16 token: HBM -> LDS by DMA, 16 bytes per lane, laid out for the transposing reads
    // Chunk p = 64 (wave + nwaves s) + lane of the LDS image holds the 8 inputs (a, c .. c + 7) with, for
    // blk = p / 8 and r = p % 8, a = 4 (blk / MT) + r / 2 and c = 16 (blk % MT) + 8 (r % 2).  Because the
    // 64-chunk base is a multiple of 8 blocks, the byte offset of that chunk in the token splits into a
    // per-lane constant (the offset for base 0) and a wave-uniform part, so each DMA costs one vector add.
    uint32_t lane_off;
    {
        const int blk = lane >> 3, r = lane & 7;
        const int a = 4 * (blk / MT) + (r >> 1), c = 16 * (blk % MT) + 8 * (r & 1);
        lane_off = 2u * (uint32_t)(a * NC + c);
    }
    auto load_token_dma = [&](int64_t t) {
        const unsigned char* xr = reinterpret_cast<const unsigned char*>(static_cast<const uint16_t*>(xv) + t * ldx);
        for (int base = wave * 64; base < nchunks; base += nwaves * 64) {
            const int b0 = base >> 3;                                    // first block of this DMA, wave-uniform
            const uint32_t uni = 2u * (uint32_t)(4 * (b0 / MT) * NC + 16 * (b0 % MT));
            const uint32_t off = lane_off + __builtin_amdgcn_readfirstlane(uni);
            // chunks past the real rows have offsets of at least 2 d, so one comparison covers both ends
            if (off < 2u * (uint32_t)d) dma16(xr, off, __builtin_amdgcn_readfirstlane(lds0 + base * 16));
        }
    };
    // fp32 token: split every input into three bf16 terms (exact sum) and store each term plane in
    // A-fragment order: fragment (ks, mt), slot (c % 16) + 16 g holds the 8 values a = 32 ks + 8 g + e of
    // column c = 16 mt + c % 16.
    auto load_token_f32 = [&](int64_t t) {
        const float* xr = static_cast<const float*>(xv) + t * ldx;
        const int units = ks_count * 4 * NC;
        for (int u = tid; u < units; u += nthreads) {
            const int c = u % NC, ag = u / NC;
            const int a0 = 8 * ag;
            uint32_t h0[8], h1[8], h2[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int i = (a0 + e) * NC + c;
                const float f = (i < d) ? xr[i] : 0.f;
                float r1, r2, r3;
                h0[e] = split_hi(f, r1);
                h1[e] = split_hi(r1, r2);
                h2[e] = split_hi(r2, r3);
            }
            const int ks = ag >> 2, gg = ag & 3, mt = c >> 4;
            unsigned char* dst = tsm + ((size_t)((ks * MT + mt) * 64 + (c & 15) + 16 * gg)) * 16;
            u32x4 p0, p1, p2;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                p0[p] = h0[2 * p] | (h0[2 * p + 1] << 16);
                p1[p] = h1[2 * p] | (h1[2 * p + 1] << 16);
                p2[p] = h2[2 * p] | (h2[2 * p + 1] << 16);
            }
            *reinterpret_cast<u32x4*>(dst) = p0;
            *reinterpret_cast<u32x4*>(dst + plane_bytes) = p1;
            *reinterpret_cast<u32x4*>(dst + 2 * plane_bytes) = p2;
        }
    };

    const int64_t t_step = MULTI ? (int64_t)gridDim.x * nwaves_hw : gridDim.x;
    int64_t t = MULTI ? (int64_t)blockIdx.x * nwaves_hw + wave_hw : blockIdx.x;
    if constexpr (!F32IN) {
        if (t < T) load_token_dma(t);       // in flight while the B fragments are fetched
    }
    // ---- once per workgroup: B fragments of P into LDS
    static_assert(KSREG == 0 || BGLOBAL, "register-resident fragments come from the table in device memory");
    u32x4 breg[TPW][KSREG > 0 ? KSREG : 1];
    if constexpr (KSREG > 0) {
#pragma unroll
        for (int ti = 0; ti < TPW; ++ti)
#pragma unroll
            for (int ks = 0; ks < KSREG; ++ks)
                breg[ti][ks] = ptable[min(wave * TPW + ti, last_tile) * kMaxKs + min(ks, ks_count - 1)][lane];
    } else if constexpr (BGLOBAL) {
        // nothing to stage
    } else if constexpr (MULTI) {
        for (int f = wave_hw; f < TPW * ks_count; f += nwaves_hw) {       // fragment f = ti ks_count + ks
            const int tile = min(f / ks_count, last_tile);
            *reinterpret_cast<u32x4*>(bsm + ((size_t)f * 64 + lane) * 16) = ptable[tile * kMaxKs + f % ks_count][lane];
        }
        lds_barrier();                      // the only workgroup barrier: every wave passes it exactly once
    } else {
#pragma unroll
        for (int ti = 0; ti < TPW; ++ti) {
            const int tile = min(wave * TPW + ti, last_tile);
            for (int ks = 0; ks < ks_count; ++ks)
                *reinterpret_cast<u32x4*>(bsm + ((size_t)(ti * ks_count + ks) * 64 + lane) * 16) = ptable[tile * kMaxKs + ks][lane];
        }
    }
    // Synchronisation among the waves that share a token: a barrier, or for a single wave only a wait for
    // its own LDS traffic (waves of a multi-token workgroup run different numbers of tokens, so they must
    // not meet at barriers inside the token loop).
    auto token_sync = [&]() {
        if constexpr (MULTI) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        else lds_barrier();
    };
    const int l4 = (lane >> 4) & 1, l5 = lane >> 5;
    const int c0 = run_start<KLOG2>(l4, l5);
    const float g7 = (float)(gamma / 7.0), g15 = (float)(gamma / 15.0);

    for (; t < T; t += t_step) {
        if constexpr (F32IN) {
            lds_barrier();                  // every wave has finished reading the previous token
            load_token_f32(t);
        } else {
            wait_all_vm();                  // this wave's part of the token (and its earlier stores) has landed
        }
        token_sync();

        // ---- base block on the matrix cores: Z^T[c][a'] = sum_a X~[a][c] P[a][a']
        f32x4 acc[TPW][MT];
        // first: the accumulators start from a literal zero; frag_of(ti): the B fragment of tile ti for this K step
        auto base_block = [&](int ks, auto first, auto frag_of) {
            constexpr bool FIRST = decltype(first)::value;
            bf16x8 bfrag[TPW];
#pragma unroll
            for (int ti = 0; ti < TPW; ++ti) bfrag[ti] = frag_of(ti);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if constexpr (!F32IN) {
                    // two transposing reads: lane (g, j = lane % 16) addresses 8 bytes of row 32 ks + 8 g + 4 h + j / 4
                    // and receives rows 32 ks + 8 g + 4 h + (0..3) of column 16 mt + j.
                    const unsigned char* p0 = tsm + ((size_t)((8 * ks + 2 * g) * MT + mt)) * 128 + 8 * l15;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 PME_AS3*)p0);
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 PME_AS3*)(p0 + MT * 128));
                    typedef __attribute__((ext_vector_type(8))) short s16x8;
                    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x8 af = __builtin_bit_cast(bf16x8, both);
#pragma unroll
                    for (int ti = 0; ti < TPW; ++ti)   // tiles beyond the block have all-zero B fragments
                        acc[ti][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            af, bfrag[ti], FIRST ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[ti][mt], 0, 0, 0);
                } else {
#pragma unroll
                    for (int sp = 0; sp < NS; ++sp) {
                        const u32x4 raw = *reinterpret_cast<const u32x4*>(
                            tsm + (size_t)sp * plane_bytes + ((size_t)((ks * MT + mt) * 64 + lane)) * 16);
                        const bf16x8 af = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
                        for (int ti = 0; ti < TPW; ++ti)
                            acc[ti][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                af, bfrag[ti], (FIRST && sp == 0) ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[ti][mt], 0, 0, 0);
                    }
                }
            }
        };
        if constexpr (KSREG > 0) {
            static_for<KSREG>([&](auto kc) {
                constexpr int KS = decltype(kc)::value;
                auto from_regs = [&](int ti) { return __builtin_bit_cast(bf16x8, breg[ti][KS]); };
                if constexpr (KS == 0) base_block(0, std::true_type{}, from_regs);
                else if (KS < ks_count) base_block(KS, std::false_type{}, from_regs);       // wave-uniform
            });
        } else {
            auto from_memory = [&](int ks) {
                return [&, ks](int ti) {
                    if constexpr (BGLOBAL)
                        return __builtin_bit_cast(bf16x8, ptable[min(wave * TPW + ti, last_tile) * kMaxKs + ks][lane]);
                    else
                        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(bsm + ((size_t)(ti * ks_count + ks) * 64 + lane) * 16));
                };
            };
            base_block(0, std::true_type{}, from_memory(0));
            for (int ks = 1; ks < ks_count; ++ks) base_block(ks, std::false_type{}, from_memory(ks));
        }

        if constexpr (!F32IN) {
            // every wave has read the token out of LDS: refill the buffer with the next token now
            token_sync();
            if (t + t_step < T) load_token_dma(t + t_step);
        }

        // ---- FWHT along c, in registers
        float v[TPW][NREG];
#pragma unroll
        for (int ti = 0; ti < TPW; ++ti) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) v[ti][mt * 4 + r] = acc[ti][mt][r];
            if ((wave * TPW + ti) * 16 < b) fwht_lane<KLOG2>(v[ti]);   // tiles beyond the block hold zeros
        }

        if constexpr (OUT == OUT_XHAT) {
            const float gf = (float)gamma;
#pragma unroll
            for (int ti = 0; ti < TPW; ++ti) {
                const int ap = (wave * TPW + ti) * 16 + l15;
                if (ap < b) {
                    float* o = xhat + t * d_e + (int64_t)ap * NC + c0;
#pragma unroll
                    for (int j = 0; j < L::RUN; ++j) o[j] = v[ti][L::reg_of_run_pos(j)] * gf;
                }
            }
        }
        if constexpr (OUT == OUT_MXFP4) {
            // ---- OCP MXFP4: one E8M0 scale per 32 consecutive outputs, E2M1 elements (round half to even,
            //      saturating) by the hardware conversion.  A lane's run of RUN outputs holds whole blocks
            //      when RUN >= 32; otherwise the block is shared with the lanes that differ in lane bit 4
            //      (and bit 5 for 2^k = 32).
            const float gf = (float)gamma;
            constexpr int PER = L::RUN >= 32 ? 32 : L::RUN;        // values of one block held by this lane
            constexpr int NBLK = L::RUN / PER;
#pragma unroll
            for (int ti = 0; ti < TPW; ++ti) {
                if ((wave * TPW + ti) * 16 >= b) continue;
                const int ap = (wave * TPW + ti) * 16 + l15;
                uint32_t words[L::RUN / 8];
                uint32_t bytes[NBLK];
#pragma unroll
                for (int blk = 0; blk < NBLK; ++blk) {
                    float amax = 0.f;
#pragma unroll
                    for (int j = 0; j < PER; j += 2)
                        amax = __builtin_fmaxf(__builtin_fmaxf(amax, __builtin_fabsf(v[ti][L::reg_of_run_pos(blk * PER + j)])),
                                               __builtin_fabsf(v[ti][L::reg_of_run_pos(blk * PER + j + 1)]));
                    if (L::RUN < 32) amax = fmaxf(amax, __shfl_xor(amax, 16));
                    if (L::RUN < 16) amax = fmaxf(amax, __shfl_xor(amax, 32));
                    bytes[blk] = mx_scale_byte(amax * gf);
                    const float X = mx_scale_value(bytes[blk]);
#pragma unroll
                    for (int wd = 0; wd < PER / 8; ++wd) {
#define PME_V(J) (v[ti][L::reg_of_run_pos(blk * PER + wd * 8 + (J))] * gf)
                        const uint32_t word = mx_pack8(PME_V(0), PME_V(1), PME_V(2), PME_V(3), PME_V(4), PME_V(5), PME_V(6), PME_V(7), X);
#undef PME_V
                        words[blk * (PER / 8) + wd] = word;
                    }
                }
                if (ap < b) {
                    uint8_t* o = qx + t * (int64_t)(d_e / 2) + (((int64_t)ap * NC + c0) >> 1);
                    if constexpr (L::RUN / 8 == 1) {
                        *reinterpret_cast<uint32_t*>(o) = words[0];
                    } else if constexpr (L::RUN / 8 == 2) {
                        *reinterpret_cast<u32x2*>(o) = u32x2{words[0], words[1]};
                    } else {
#pragma unroll
                        for (int wd = 0; wd < L::RUN / 8; wd += 4)
                            *reinterpret_cast<u32x4*>(o + 4 * wd) = u32x4{words[wd], words[wd + 1], words[wd + 2], words[wd + 3]};
                    }
                    const bool owner = (L::RUN >= 32) || (L::RUN == 16 && l4 == 0) || (l4 == 0 && l5 == 0);
                    if (owner) {
                        uint8_t* eo = ex + t * (int64_t)(d_e / 32) + (((int64_t)ap * NC + c0) >> 5);
#pragma unroll
                        for (int blk = 0; blk < NBLK; ++blk) eo[blk] = (uint8_t)bytes[blk];
                    }
                }
            }
        }
        if constexpr (OUT == OUT_SYM || OUT == OUT_ASYM) {
        // ---- per-token range
        float hi = 0.f, lo = 0.f;
        if constexpr (OUT == OUT_ASYM) {
#pragma unroll
            for (int ti = 0; ti < TPW; ++ti)
#pragma unroll
                for (int i = 0; i < NREG; i += 2) {       // v_max3_f32 / v_min3_f32: one instruction per element in all
                    hi = __builtin_fmaxf(__builtin_fmaxf(hi, v[ti][i]), v[ti][i + 1]);
                    lo = __builtin_fminf(__builtin_fminf(lo, v[ti][i]), v[ti][i + 1]);
                }
            lo = wave_min(lo);
        } else {
#pragma unroll
            for (int ti = 0; ti < TPW; ++ti)
#pragma unroll
                for (int i = 0; i < NREG; i += 2) hi = __builtin_fmaxf(__builtin_fmaxf(hi, __builtin_fabsf(v[ti][i])), __builtin_fabsf(v[ti][i + 1]));
        }
        hi = wave_max(hi);
        if (nwaves > 1) {
            // the scratch is reused per token: the barrier of the matrix phase separates the tokens
            if (lane == 0) { red[wave] = hi; red[kMaxWaves + wave] = lo; }
            lds_barrier();
            for (int w = 0; w < nwaves; ++w) {
                hi = fmaxf(hi, red[w]);
                lo = fminf(lo, red[kMaxWaves + w]);
            }
        }

        float s = 1.f, rinv = 0.f;
        int z = 0;
        if constexpr (OUT == OUT_SYM) {
            if (hi > 0.f) {
                s = hi * g7;                      // absmax * gamma / 7
                rinv = 7.f * __builtin_amdgcn_rcpf(hi);
            }
            if (tid == 0) sx[t] = s;
        } else {
            if (hi > lo) {
                // fp32 like the symmetric case: scale = range * fp32(gamma / 15), codes from u * (15 / range)
                const float range = hi - lo;
                s = range * g15;
                rinv = 15.f * __builtin_amdgcn_rcpf(range);
                z = (int)__builtin_rintf(-lo * rinv);
                z = min(15, max(0, z));
            }
            if (tid == 0) { sx[t] = s; zx[t] = z; }
        }

        // ---- round, pack, store.
        // fma(u, rinv, 1.5 * 2^23 + 8) has the bit pattern C + e with C = 0x4B400000 and e = rne(u * rinv) + 8
        // in [1, 15].  Eight of them are combined by Horner steps acc = (acc << 4) + bits; the digits are
        // non-negative, so no carries cross nibbles, and the accumulated constant C * 0x11111111 is
        // subtracted once.  e ^ 8 is the 4-bit two's-complement code.
        constexpr uint32_t kC = 0x4B400000u;
        constexpr uint32_t kCsum = kC * 0x11111111u;
#pragma unroll
        for (int ti = 0; ti < TPW; ++ti) {
            if ((wave * TPW + ti) * 16 >= b) continue;      // wave-uniform: nothing to store for this tile
            const int ap = (wave * TPW + ti) * 16 + l15;
            uint32_t words[L::RUN / 8];
#pragma unroll
            for (int wd = 0; wd < L::RUN / 8; ++wd) {
                if constexpr (OUT == OUT_SYM) {
                    uint32_t accw = 0;
#pragma unroll
                    for (int nb = 7; nb >= 0; --nb) {
                        const float f = __builtin_fmaf(v[ti][L::reg_of_run_pos(wd * 8 + nb)], rinv, 12582920.f);
                        accw = (accw << 4) + __float_as_uint(f);
                    }
                    words[wd] = (accw - kCsum) ^ 0x88888888u;
                } else {
                    // the zero point rides in the rounding constant (rne(u rinv + z) = rne(u rinv) + z), the clamp
                    // to [0, 15] is one median-of-three on the float, then the same Horner packing
                    const float cz = 12582912.f + (float)z;
                    uint32_t accw = 0;
#pragma unroll
                    for (int nb = 7; nb >= 0; --nb) {
                        float f = __builtin_fmaf(v[ti][L::reg_of_run_pos(wd * 8 + nb)], rinv, cz);
                        f = __builtin_amdgcn_fmed3f(f, 12582912.f, 12582927.f);
                        accw = (accw << 4) + __float_as_uint(f);
                    }
                    words[wd] = accw - kCsum;
                }
            }
            if (ap < b) {
                uint8_t* o = qx + t * (int64_t)(d_e / 2) + (((int64_t)ap * NC + c0) >> 1);
                if constexpr (L::RUN / 8 == 1) {
                    *reinterpret_cast<uint32_t*>(o) = words[0];
                } else if constexpr (L::RUN / 8 == 2) {
                    *reinterpret_cast<u32x2*>(o) = u32x2{words[0], words[1]};
                } else {
#pragma unroll
                    for (int wd = 0; wd < L::RUN / 8; wd += 4)
                        *reinterpret_cast<u32x4*>(o + 4 * wd) = u32x4{words[wd], words[wd + 1], words[wd + 2], words[wd + 3]};
                }
            }
        }
        }   // int4 outputs
    }
    wait_all_vm();
}

// Workgroups of `threads` threads and `lds` bytes of dynamic LDS that one compute unit holds at once, as the runtime
// computes it from the kernel's registers and LDS (a host-side calculation; cached per kernel for the last few
// launch shapes).  At least 1.
template <class K> int resident_workgroups(K kern, int threads, size_t lds) {
    struct Entry { int threads; size_t lds; int n; };
    static std::mutex mu;
    static std::vector<Entry> cache;
    std::lock_guard<std::mutex> lock(mu);
    for (const Entry& e : cache)
        if (e.threads == threads && e.lds == lds) return e.n;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void*)kern, threads, lds) != hipSuccess || n < 1) n = 1;
    if (cache.size() < 64) cache.push_back(Entry{threads, lds, n});
    return n;
}

template <int KLOG2, int TPW, bool F32IN, int OUT, bool BGLOBAL = false, int KSREG = 0>
pme_status launch_out(const RotateArgs& a, int ks, int nwaves) {
    using L = Layout<KLOG2>;
    constexpr int NS = F32IN ? 3 : 1;
    const size_t lds = (size_t)NS * ks * L::MT * 1024 + (BGLOBAL ? 0 : (size_t)nwaves * TPW * ks * 1024);
    // 160 KB per workgroup, less the kernel's static LDS rounded up to the dynamic part's 1 KB alignment
    constexpr size_t kMaxDynLds = 160 * 1024 - 1024;
    if (lds > kMaxDynLds || nwaves > max_waves<KLOG2, TPW>()) return PME_ERR_UNSUPPORTED_PATH;
    if (KSREG > 0 && ks > KSREG) return PME_ERR_UNSUPPORTED_PATH;
    if (a.dry) return PME_OK;
    const int rows = (int)((a.d + L::NC - 1) >> KLOG2);
    pme_status st = PME_OK;
    const Fragment* ptable = fragment_table(a.b >> a.fold, a.fold, rows, a.stream, &st);
    if (!ptable) return st;
    auto kern = k_rotate_mfma<KLOG2, TPW, F32IN, OUT, false, BGLOBAL, KSREG>;
    // the same kernel runs with different LDS sizes (they follow the shape): allow the largest one accepted above
    static std::atomic<uint32_t> done;
    if (lds > 48 * 1024 && allow_dynamic_lds(kern, (int)kMaxDynLds, done) != PME_OK) return PME_ERR_HIP;
    // Persistent grid: as many workgroups as fit on the 256 compute units at once: LDS, and 16 waves per
    // compute unit (measured: 12 left memory latency exposed -- 8448 .. 9728, 18432 and 22016 ran 14-20 % slower
    // -- and 20 is past what the registers admit); the four-wave workgroups of 2^k = 256 (15360) are the
    // exception, 10 % faster at three per compute unit than at four.
    int occ = (int)((160 * 1024) / (lds + 1024));
    occ = std::min(occ, (KLOG2 == 8 && nwaves == 4 ? 12 : 16) / nwaves);
    occ = std::max(1, std::min(occ, 8));
    // never more workgroups than are resident at once (registers may admit fewer than LDS and the wave count do):
    // a persistent grid larger than that would run in two uneven rounds
    occ = std::min(occ, resident_workgroups(kern, 64 * nwaves, lds));
    const unsigned grid = (unsigned)std::min<int64_t>(a.T, 256 * (int64_t)occ);
    const double gamma = 1.0 / sqrt((double)a.d_e);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * nwaves), lds, a.stream, a.x, a.ldx, (int)a.T, (int)a.d,
                       (int)a.d_e, a.b, ks, ptable, gamma, a.qx, a.sx, a.zx, a.ex, a.xhat);
    return hip_status(hipGetLastError());
}

// Multi-token workgroups of kMultiWaves waves (bf16 input, a token per wave).
constexpr int kMultiWaves = 4;
// KSREG > 0: the fragments live in each wave's registers (read once from the table) instead of shared LDS.
template <int KLOG2, int TPW, int OUT, int KSREG>
pme_status launch_multi_out(const RotateArgs& a, int ks) {
    using L = Layout<KLOG2>;
    const size_t lds = (size_t)kMultiWaves * ks * L::MT * 1024 + (KSREG > 0 ? 0 : (size_t)TPW * ks * 1024);
    constexpr size_t kMaxDynLds = 160 * 1024 - 1024;
    if (lds > kMaxDynLds) return PME_ERR_UNSUPPORTED_PATH;
    if (a.dry) return PME_OK;
    const int rows = (int)((a.d + L::NC - 1) >> KLOG2);
    pme_status st = PME_OK;
    const Fragment* ptable = fragment_table(a.b >> a.fold, a.fold, rows, a.stream, &st);
    if (!ptable) return st;
    auto kern = k_rotate_mfma<KLOG2, TPW, false, OUT, true, (KSREG > 0), KSREG>;
    static std::atomic<uint32_t> done;
    if (lds > 48 * 1024 && allow_dynamic_lds(kern, (int)kMaxDynLds, done) != PME_OK) return PME_ERR_HIP;
    int occ = (int)((160 * 1024) / (lds + 1024));
    occ = std::max(1, std::min(occ, 12 / kMultiWaves));
    const int64_t groups = (a.T + kMultiWaves - 1) / kMultiWaves;
    const unsigned grid = (unsigned)std::min<int64_t>(groups, 256 * (int64_t)occ);
    const double gamma = 1.0 / sqrt((double)a.d_e);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * kMultiWaves), lds, a.stream, a.x, a.ldx, (int)a.T, (int)a.d,
                       (int)a.d_e, a.b, ks, ptable, gamma, a.qx, a.sx, a.zx, a.ex, a.xhat);
    return hip_status(hipGetLastError());
}
template <int KLOG2, int TPW, int KSREG>
pme_status launch_multi_ks(const RotateArgs& a, int ks) {
    if (a.xhat) return launch_multi_out<KLOG2, TPW, OUT_XHAT, KSREG>(a, ks);
    if (a.ex) return launch_multi_out<KLOG2, TPW, OUT_MXFP4, KSREG>(a, ks);
    if (a.zx) return launch_multi_out<KLOG2, TPW, OUT_ASYM, KSREG>(a, ks);
    return launch_multi_out<KLOG2, TPW, OUT_SYM, KSREG>(a, ks);
}
template <int KLOG2, int TPW>
pme_status launch_multi(const RotateArgs& a, int ks) {
    // up to 64 real base rows (two K steps): 10 fragments per wave fit in registers, 5 % faster than shared LDS
    if (ks <= 2) return launch_multi_ks<KLOG2, TPW, 2>(a, ks);
    return launch_multi_ks<KLOG2, TPW, 0>(a, ks);
}

template <int KLOG2, int TPW, bool F32IN, bool BGLOBAL = false, int KSREG = 0>
pme_status launch_one(const RotateArgs& a, int ks, int nwaves) {
    if (a.xhat) return launch_out<KLOG2, TPW, F32IN, OUT_XHAT, BGLOBAL, KSREG>(a, ks, nwaves);
    if (a.ex) return launch_out<KLOG2, TPW, F32IN, OUT_MXFP4, BGLOBAL, KSREG>(a, ks, nwaves);
    if (a.zx) return launch_out<KLOG2, TPW, F32IN, OUT_ASYM, BGLOBAL, KSREG>(a, ks, nwaves);
    return launch_out<KLOG2, TPW, F32IN, OUT_SYM, BGLOBAL, KSREG>(a, ks, nwaves);
}

int g_tpw_override = 0;
int g_multi_override = -1;     // experiments: 0 / 1 force the multi-token variant off / on where it applies

}  // namespace

void set_rotate_tpw_override(int tpw) { g_tpw_override = tpw; }

pme_status launch_rotate_mfma(const RotateArgs& in) {
    // Shapes covered: 2^k >= 32; in-register butterflies span at most 512 columns, so for larger 2^k the
    // first stages are folded into the base block (order b 2^fold), which the matrix cores apply: the kernel
    // sees the same transform as a block of that order times fewer columns.
    // bf16 input is copied to LDS in 16-byte pieces, so d, the row pitch and the base address must be
    // multiples of 8 elements; code rows must be 16-byte aligned.
    RotateArgs a = in;
    // Fold butterfly stages into the base block: down to 2^k = 128 (or 256) while the block's order stays within
    // 80 -- lighter waves and more of them per token than at 2^k = 512 (10240 = 20 x 512 runs as 80 x 128: 21 ->
    // 14 us for 2048 tokens; 4096 as 32 x 128: 14.5 -> 6.2 us) -- else down to the 512 columns the registers hold.
    for (int target = 7; target <= 9 && a.fold == 0; ++target) {
        if (a.k <= target) break;
        const int f = a.k - target;
        const int64_t order = (int64_t)a.b << f;
        if (f > 8 || order > (target < 9 ? 80 : 16 * kMaxTiles)) continue;
        a.fold = f;
        a.b = (int)order;
        a.k = target;
    }
    if (a.k > 9) return PME_ERR_UNSUPPORTED_PATH;
    if (a.k < 5) return PME_ERR_UNSUPPORTED_PATH;
    const bool f32 = a.xt == PME_F32;
    if (!f32 && ((a.d & 7) || (a.ldx & 7) || (reinterpret_cast<uintptr_t>(a.x) & 15))) return PME_ERR_UNSUPPORTED_PATH;
    if (a.qx && (reinterpret_cast<uintptr_t>(a.qx) & 15)) return PME_ERR_UNSUPPORTED_PATH;
    const int nc = 1 << a.k;
    const int rows = (int)((a.d + nc - 1) >> a.k);
    const int ks = (rows + 31) / 32;
    const int nt = (a.b + 15) / 16;
    if (ks > kMaxKs || nt > kMaxTiles) return PME_ERR_UNSUPPORTED_PATH;
    // a'-tiles per wave: bounded by registers (4 * 2^k / 16 accumulators per tile); fewer tiles per wave
    // mean more, lighter waves per token, which measured faster from 2^k = 128 up.
    int tpw;
    switch (a.k) {
        case 5: tpw = 5; break;
        case 6: tpw = 3; break;
        case 7: tpw = 2; break;
        default: tpw = 1; break;
    }
    // few tokens: spread a token over as many waves as it has tiles
    if (a.T < 512 && a.k <= 8) tpw = 1;
    if (g_tpw_override > 0) tpw = g_tpw_override;
    // P fragments read from the table in device memory instead of LDS:
    //  * 2^k = 64 with 8 tiles or more (orders 132 .. 152: 8448, 8960, 9728): staging nt ks KB of fragments
    //    leaves room for only two workgroups per compute unit; without it the kernel measured 18 % faster;
    //  * the order-312 and order-344 blocks (19968 = 312 x 64, 22016 = 344 x 64): 20 and 22 column tiles on 7
    //    and 8 waves, about 150 KB of fragments that do not fit in LDS beside the token at all;
    //  * 2^k = 128 (8704): 4 % faster.
    // Where a wave's fragments are few (TPW x K steps <= 8 registers of 16 bytes), it reads them once and keeps
    // them in registers for all its tokens: another 3-6 % (8448 .. 9728, 8704, 15360).
    if (!f32 && g_tpw_override == 0) {
        if (a.k == 6 && nt >= 8) {
            // from about 3000 tokens three tiles per wave (three waves per token, five tokens in flight per compute
            // unit) beat two (8448 .. 9728: 5-11 % at 4096 and 8192 tokens; 1-4 % slower at 2048)
            if (nt <= 16 && ks <= 4 && a.T >= 3072) return launch_one<6, 3, false, true, 4>(a, ks, (nt + 2) / 3);
            // a handful of tokens (decode): one tile per wave, nine or ten waves per token; the kernel is a chain of
            // latencies there and the lighter waves shorten it (8448, 8 tokens: 4.1 -> 3.8 us)
            if (nt <= kMaxWaves && ks <= 4 && a.T <= 64) return launch_one<6, 1, false, true, 4>(a, ks, nt);
            if (nt <= 2 * kMaxWaves && ks <= 4) return launch_one<6, 2, false, true, 4>(a, ks, (nt + 1) / 2);
            // beyond 16 tiles three per wave: 7 waves for the order-312 block, so that two workgroups share a compute
            // unit (19968: 42 -> 36 us for 2048 tokens against 10 waves of two tiles)
            if (nt <= 16) return launch_one<6, 2, false, true>(a, ks, (nt + 1) / 2);
            return launch_one<6, 3, false, true>(a, ks, (nt + 2) / 3);
        }
        if (a.k == 7 && tpw == 2 && ks <= 2) return launch_one<7, 2, false, true, 2>(a, ks, (nt + 1) / 2);
        if (a.k == 7 && tpw == 2) return launch_one<7, 2, false, true>(a, ks, (nt + 1) / 2);
        if (a.k == 8 && tpw == 1 && ks <= 2) return launch_one<8, 1, false, true, 2>(a, ks, nt);
    }
    const int nwaves = (nt + tpw - 1) / tpw;
    if (nwaves > kMaxWaves) return PME_ERR_UNSUPPORTED_PATH;
    // 2^k = 32 with a block of at most 80: the token is one wave's work and only a few KB
    const bool multi = g_multi_override >= 0 ? g_multi_override == 1 : a.T >= 1024;
    if (!f32 && a.k == 5 && tpw == 5 && nwaves == 1 && multi) return launch_multi<5, 5>(a, ks);
#define PME_ROT(K, TP)                                                             \
    if (a.k == K && tpw == TP)                                                     \
        return f32 ? launch_one<K, TP, true>(a, ks, nwaves) : launch_one<K, TP, false>(a, ks, nwaves);
    PME_ROT(5, 5) PME_ROT(5, 3) PME_ROT(5, 1)
    PME_ROT(6, 3) PME_ROT(6, 2) PME_ROT(6, 1)
    PME_ROT(7, 3) PME_ROT(7, 2) PME_ROT(7, 1)
    PME_ROT(8, 2) PME_ROT(8, 1)
    PME_ROT(9, 1)
#undef PME_ROT
    return PME_ERR_UNSUPPORTED_PATH;
}

}  // namespace pme
