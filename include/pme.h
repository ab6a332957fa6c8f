/*
 * pme.h - C ABI of the expanded W4A4 linear layer for MI355X (gfx950).
 *
 * The operation is the inference path of post-training model expansion
 * (paper Section 3): activations X (T x d) are rotated online by the expanded
 * Hadamard matrix H_hat (d x d_e, the first d rows of a d_e x d_e Hadamard matrix
 * scaled by gamma = 1/sqrt(d_e)), X_hat = X H_hat, quantized per token, and multiplied
 * by the offline-expanded, quantized weights Q(W_hat), W_hat = H_hat^T W, so that the
 * layer computes Q(X_hat) Q(W_hat) ~ X W.  Paper notation D, N, M, N' corresponds to
 * T, d, d_e, N here.
 *
 * The Hadamard matrix of order d_e = b * 2^k is H = P_b (x) S_{2^k}: a Paley type-I
 * block of order b (b - 1 a prime congruent to 3 mod 4, or 7^3; b = 1 for a pure power
 * of two; supported: 1, 12, 20, 60, 68, 72, 132, 140, 152, 312, 344) Kronecker the
 * natural-order Sylvester matrix; matrix index i = a * 2^k + c.
 * Section 4 only asks for a deterministic Hadamard matrix and does not fix the
 * construction; pme_base_block exports the block actually used.
 *
 * Conventions shared by every entry point unless stated otherwise:
 *  - Pointers named in the comments as DEVICE are HIP device memory owned by the
 *    caller.  The library never allocates, frees or synchronises; every call only
 *    enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = default
 *    stream) and returns.  One exception: the first rotation of a new shape (d, d_e) on a device fills a
 *    table of base-block fragments in library-owned device memory (a static pool of 16 MB per device, 7 to
 *    154 KB per shape, kept for the life of the process) and waits for that small kernel once; run a shape
 *    once before capturing it in a HIP graph (under capture such a first call returns PME_ERR_COLD_SHAPE
 *    and enqueues nothing).
 *  - Arguments are validated on the host before any HIP call.  A status other than
 *    PME_OK means nothing was launched (PME_ERR_HIP excepted: a launch was refused by
 *    the runtime); the fused pme_expanded_linear* calls ask both of their stages whether a
 *    kernel takes the shape before they launch the first.  No C++ exception crosses this boundary.
 *  - Packed int4: byte j/2 of a row holds code j (even j) in its low nibble and code
 *    j+1 in its high nibble, each a 4-bit two's-complement integer (unsigned 0..15 for
 *    the asymmetric activation variant).
 *  - Rows of packed codes are dense: the row pitch is d_e / 2 bytes.
 *  - Outputs must not alias inputs.
 *  - Size limits: T and N below 2^31, d_e at most 2^20 (PME_ERR_SHAPE beyond).  Operands of any byte size within
 *    those limits are accepted; a GEMM whose packed activations or weights exceed 4 GiB is enqueued as several
 *    launches over slices of tokens or output channels, with the same results.  The matrix-core int4 GEMMs hold
 *    256 x the exact sum in int32 and take d_e < 2^17 (256 * 64 * d_e < 2^31); from d_e = 2^17 on the plain-ALU
 *    kernel runs (PME_ERR_UNSUPPORTED_PATH if the matrix-core path was forced).
 */
#ifndef PME_H
#define PME_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PME_OK = 0,
    PME_ERR_NULL = 1,               /* a required pointer is NULL */
    PME_ERR_SHAPE = 2,              /* negative / inconsistent sizes, d > d_e, odd d_e, pitch too small */
    PME_ERR_UNSUPPORTED_ORDER = 3,  /* d_e is not b * 2^k with a supported base order b */
    PME_ERR_ALIGN = 4,              /* pointer or pitch alignment requirement violated */
    PME_ERR_WORKSPACE = 5,          /* workspace too small */
    PME_ERR_DTYPE = 6,              /* unknown pme_dtype */
    PME_ERR_HIP = 7,                /* the HIP runtime refused a launch */
    PME_ERR_UNSUPPORTED_PATH = 8,   /* no kernel path (or not the one forced with pme_set_path) runs this shape:
                                       e.g. a token of more than about 40000 expanded features whose block the
                                       matrix-core kernel does not take */
    PME_ERR_COLD_SHAPE = 9          /* the first rotation of this shape on this device has to fill its base-block
                                       table and wait for it, which cannot happen while `stream` is being captured
                                       into a HIP graph: nothing was enqueued and the capture is intact; make one
                                       call of the shape outside the capture first */
} pme_status;

typedef enum { PME_F32 = 0, PME_BF16 = 1 } pme_dtype;

/* Kernel-path selector (test / benchmark hook, process-wide, not thread-safe). */
typedef enum {
    PME_PATH_AUTO = 0,     /* MFMA kernels where the shape allows, generic kernels otherwise */
    PME_PATH_GENERIC = 1,  /* plain-ALU kernels for every shape */
    PME_PATH_MFMA = 2      /* MFMA kernels or PME_ERR_UNSUPPORTED_PATH */
} pme_path;

/*
 * Online expansion + rotation + per-token symmetric int4 quantization
 * (Section 3: X_hat = X H_hat; Section 4: per-token activation quantizer, taken
 * symmetric here: scale = absmax / 7, round half to even, codes in [-7, 7]).
 *   x   DEVICE [T, d] row-major, element type xt, ldx elements between rows (ldx >= d).
 *   qx  DEVICE out [T, d_e / 2] packed int4 codes.   sx  DEVICE out [T] fp32 scales
 *       (x_hat[t][j] ~ sx[t] * code[t][j]; an all-zero token gets scale 1, codes 0).
 * Alignment: x to its element size, qx to 4 bytes (16 for the MFMA path), sx to 4.
 * T == 0 is a no-op returning PME_OK.
 */
pme_status pme_hadamard_expand_quant(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                     int64_t d_e, uint8_t* qx, float* sx, void* stream);

/*
 * Same rotation, per-token asymmetric uint4 quantization (the paper's Section 4 setting):
 * lo = min(min_j, 0), hi = max(max_j, 0), scale = (hi - lo) / 15, zero point
 * z = rne(-lo / scale) in [0, 15], code = clamp(rne(x / scale) + z, 0, 15).
 *   zx  DEVICE out [T] int32 zero points.  Other arguments as above (codes are unsigned).
 */
pme_status pme_hadamard_expand_quant_asym(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                          int64_t d_e, uint8_t* qx, float* sx, int32_t* zx, void* stream);

/*
 * int4 x int4 GEMM with fused dequantisation (Section 3: Q(X_hat) Q(W_hat); Section 4:
 * per-token activation scale, per-output-channel weight scale):
 *   y[t][n] = bf16( (sum_j qx[t][j] * qw[n][j]) * sx[t] * sw[n] ).
 *   qx DEVICE [T, d_e/2], sx DEVICE [T]; qw DEVICE [N, d_e/2] (one row of d_e codes per
 *   output channel, i.e. the transpose of the paper's W_hat), sw DEVICE [N].
 *   y  DEVICE out [T, N] bf16 row-major, ldy elements between rows (ldy >= N).
 * The sum is exact int32 (|sum| <= 64 * d_e).  Alignment: qx, qw to 4 bytes (16 for the
 * MFMA path), y to 2 bytes.  T == 0 or N == 0 is a no-op.  The call needs no workspace:
 * partial sums never leave registers and LDS.
 */
pme_status pme_w4a4_gemm(const uint8_t* qx, const float* sx, const uint8_t* qw, const float* sw,
                         int64_t T, int64_t d_e, int64_t N, void* y_bf16, int64_t ldy, void* stream);

/*
 * Asymmetric-activation variant: codes qx are unsigned with zero point zx[t];
 *   y[t][n] = bf16( (sum_j qx[t][j] qw[n][j] - zx[t] * wsum[n]) * sx[t] * sw[n] ),
 *   wsum DEVICE [N] int32 = sum_j qw[n][j] (see pme_weight_rowsum).
 */
pme_status pme_w4a4_gemm_asym(const uint8_t* qx, const float* sx, const int32_t* zx, const uint8_t* qw,
                              const float* sw, const int32_t* wsum, int64_t T, int64_t d_e, int64_t N,
                              void* y_bf16, int64_t ldy, void* stream);

/* Offline companion of the asymmetric quantizer of Section 4: wsum[n] = sum_j qw[n][j] for packed signed weight
 * codes, the factor of the zero-point correction above.  qw DEVICE [N, d_e/2], wsum DEVICE out [N]. */
pme_status pme_weight_rowsum(const uint8_t* qw, int64_t N, int64_t d_e, int32_t* wsum, void* stream);

/*
 * The whole expanded layer in one call (Section 3: the inference-time product Q(X H_hat) Q(H_hat^T W), with the
 * per-token / per-channel scales of Section 4): pme_hadamard_expand_quant followed by
 * pme_w4a4_gemm, the codes and scales passing through `workspace`
 * (DEVICE, 256-byte aligned, at least pme_workspace_bytes(T, d, d_e, N) bytes; contents undefined afterwards).
 * Arguments as in the two calls.  PME_ERR_WORKSPACE if the workspace is too small.
 */
pme_status pme_expanded_linear(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                               int64_t d_e, const uint8_t* qw, const float* sw, int64_t N,
                               void* y_bf16, int64_t ldy, void* workspace, size_t workspace_bytes,
                               void* stream);

/*
 * pme_expanded_linear for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * pme_expanded_linear, minus the workspace: the quantized activations pass through a static array in the
 * library's device image, PME_STATIC_SCRATCH_BYTES per GPU, held until the process ends.  The call allocates and
 * frees nothing and enqueues the same kernels.  PME_ERR_WORKSPACE (nothing launched) if
 * pme_workspace_bytes(T, d, d_e, N) exceeds PME_STATIC_SCRATCH_BYTES, i.e. T * d_e / 2 above roughly 16 Mi.
 * Every call on a GPU shares that GPU's array: calls that can overlap on one GPU (different streams, or threads)
 * race on it; calls on one stream do not.  Nothing in the array needs clearing between calls (the rotation writes
 * all the GEMM reads).  The first call on a device looks the array's address up once, which is when the runtime
 * places the array in that device's memory (and, like every rotation, the first call of a new shape fills its
 * base-block table): make one call per shape before capturing a graph or entering a region that must not allocate.
 */
#define PME_STATIC_SCRATCH_BYTES (16u << 20)
pme_status pme_expanded_linear_static(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                      int64_t d_e, const uint8_t* qw, const float* sw, int64_t N,
                                      void* y_bf16, int64_t ldy, void* stream);

/*
 * The same with the paper's activation quantizer (Section 4: per-token asymmetric int4):
 * pme_hadamard_expand_quant_asym followed by pme_w4a4_gemm_asym; wsum DEVICE [N] from pme_weight_rowsum.
 * Codes, scales and zero points pass through `workspace` (same size and alignment as above).
 */
pme_status pme_expanded_linear_asym(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                    int64_t d_e, const uint8_t* qw, const float* sw, const int32_t* wsum,
                                    int64_t N, void* y_bf16, int64_t ldy, void* workspace,
                                    size_t workspace_bytes, void* stream);

/*
 * Offline weight side (Section 3: W_hat = H_hat^T W; Section 4: per-channel symmetric int4, here by
 * round-to-nearest): expands and quantizes a weight matrix into the qw / sw operands of pme_w4a4_gemm.
 *   wt  DEVICE [N, d] row-major (one row of d input weights per output channel, i.e. W^T of the paper's
 *       d x N matrix), element type wtype, ldw elements between rows.
 *   qw  DEVICE out [N, d_e / 2] packed int4,  sw  DEVICE out [N] fp32 (scale = absmax / 7 per channel).
 * Row n of W_hat^T is the rotation of row n of W^T, so this is the activation transform applied to the
 * rows of wt; same alignment rules as pme_hadamard_expand_quant.  GPTQ-style calibration is not done.
 */
pme_status pme_expand_quantize_weights(const void* wt, pme_dtype wtype, int64_t N, int64_t d, int64_t ldw,
                                       int64_t d_e, uint8_t* qw, float* sw, void* stream);

/*
 * OCP MXFP4 variants (Section 4, second setting: MXFP4 for weights and activations, one E8M0 scale per
 * group of 32 elements).  Element format FP4 E2M1 (magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6), block scale
 * 2^(byte - 127) with byte - 127 = floor(log2(block absmax)) - 2, elements rounded half to even and
 * saturating at +-6, an all-zero block takes byte 0.  d_e must be a multiple of 32.
 *   qx DEVICE out [T, d_e/2] packed E2M1 codes (even index in the low nibble),
 *   ex DEVICE out [T, d_e/32] E8M0 bytes.
 * Applied to the rows of a [N, d] weight matrix (W^T) the same call is the offline weight side.
 */
pme_status pme_hadamard_expand_quant_mxfp4(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                           int64_t d_e, uint8_t* qx, uint8_t* ex, void* stream);

/* y[t][n] = bf16(sum over blocks of 32 of 2^(ex-127) 2^(ew-127) sum_i P_x,i P_w,i), fp32 accumulation.
 *   qx [T, d_e/2], ex [T, d_e/32], qw [N, d_e/2], ew [N, d_e/32] DEVICE; y DEVICE out [T, N] bf16, pitch ldy. */
pme_status pme_mxfp4_gemm(const uint8_t* qx, const uint8_t* ex, const uint8_t* qw, const uint8_t* ew,
                          int64_t T, int64_t d_e, int64_t N, void* y_bf16, int64_t ldy, void* stream);

/* The whole MXFP4 expanded layer: the two calls above, codes and scale bytes passing through `workspace`
 * (DEVICE, 256-byte aligned, at least pme_workspace_bytes bytes). */
pme_status pme_expanded_linear_mxfp4(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                     int64_t d_e, const uint8_t* qw, const uint8_t* ew, int64_t N,
                                     void* y_bf16, int64_t ldy, void* workspace, size_t workspace_bytes,
                                     void* stream);

/* Bytes of workspace the pme_expanded_linear* calls need for the quantized activations of Section 3's Q(X H_hat):
 * packed codes [T, d_e/2], per-token scales (or MXFP4 scale bytes) and zero points, each part 256-byte aligned
 * (one size serves all three calls; 0 on invalid sizes).  N is accepted for symmetry and does not enter. */
size_t pme_workspace_bytes(int64_t T, int64_t d, int64_t d_e, int64_t N);

/* ---- parity / debug exports ---- */

/* X_hat = X H_hat itself (Section 3; gamma = 1/sqrt(d_e) applied), fp32, unquantized: xhat DEVICE out
 * [T, d_e] dense.  x as in pme_hadamard_expand_quant.  Applied to the rows of W^T it is W_hat^T. */
pme_status pme_hadamard_expand_f32(const void* x, pme_dtype xt, int64_t T, int64_t d, int64_t ldx,
                                   int64_t d_e, float* xhat, void* stream);

/* The raw int32 accumulators of Section 3's Q(X_hat) Q(W_hat), before any scale: acc[t][n] = sum_j qx[t][j] qw[n][j]
 * for signed codes, exact.  qx DEVICE [T, d_e/2], qw DEVICE [N, d_e/2], acc DEVICE out [T, N] dense. */
pme_status pme_w4a4_gemm_i32(const uint8_t* qx, const uint8_t* qw, int64_t T, int64_t d_e, int64_t N,
                             int32_t* acc, void* stream);

/* The factorisation of the expanded size M = d_e of Section 3 that the Hadamard matrix is built from:
 * d_e = b * 2^k with the smallest supported b; b, k HOST out.  PME_ERR_UNSUPPORTED_ORDER if none. */
pme_status pme_factor_order(int64_t d_e, int32_t* b, int32_t* k);

/* The +-1 Paley block P_b of the Hadamard matrix H = P_b (x) S_{2^k} behind Section 3's H_hat (Section 4 leaves the
 * construction open), row-major b x b, written to HOST memory out_bxb (b * b bytes).  P = I + [[0, 1^T], [-1, Q]],
 * Q[i][j] = chi(x_i - x_j) over GF(b - 1).  PME_ERR_UNSUPPORTED_ORDER for an order not in the list above. */
pme_status pme_base_block(int64_t b, int8_t* out_bxb);

/* Input preparation for the weight operand (Section 4: int4 weights; two codes per byte as stated under
 * "Packed int4" above): codes DEVICE [rows, K] int8 in [-8, 7] (only the low 4 bits are kept), packed DEVICE out
 * [rows, K/2].  K even, both dense. */
pme_status pme_pack_int4(const int8_t* codes, int64_t rows, int64_t K, uint8_t* packed, void* stream);

/* ---- measurement helpers ---- */

/* Plain device copy of `bytes` (multiple of 16) from src to dst, both DEVICE and 16-byte aligned, four 16-byte
 * loads in flight per lane: the known-size kernel that calibrates the profiler's HBM byte counters and gives the
 * measured read + write streaming rate. */
pme_status pme_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Read-only stream of `bytes` (multiple of 16) from src (DEVICE, 16-byte aligned), same load pattern as the copy:
 * the measured ceiling for a stage that mostly reads, as rotate + quantize does (four fifths of its bytes).
 * sink: DEVICE out, at least 2048 * 256 uint32 (one checksum per lane, the probe's only writes). */
pme_status pme_probe_read(const void* src, size_t bytes, uint32_t* sink, size_t sink_elems, void* stream);

/* Enqueues a kernel that does nothing (one wave): timing a chain of them gives the cost of a dependent launch,
 * the floor under a layer that is two tiny kernels, as the decode shape is. */
pme_status pme_probe_launch(void* stream);

/* Back-to-back independent matrix-core instructions, nothing else in the loop: the measured ceiling the
 * GEMMs are priced against next to the published peak.  kind 0: v_mfma_i32_32x32x32_i8 (the int4 path's
 * instruction), kind 1: v_mfma_scale_f32_32x32x64_f8f6f4 on FP4 operands (the MXFP4 path's), both on near-constant
 * operands; kinds 2 and 3: the same two instructions on pseudo-random codes (for int8 the bytes the int4 GEMM
 * feeds the pipe: a random nibble times 16), whose rate is lower because the pipe is power-limited (iters is
 * rounded up to a multiple of 4 for these two).  Launches 512
 * workgroups of 256 threads, each wave issuing 4 * iters instructions; out: DEVICE int32, at least
 * 512 * 256 elements (a checksum that keeps the loop alive); *ops (HOST, may be null) receives the operation
 * count of one launch (2 per multiply-add).  PME_ERR_DTYPE for another kind, PME_ERR_SHAPE for a short
 * buffer or iters outside [0, 2^24]. */
pme_status pme_probe_mfma(int kind, int32_t* out, size_t out_elems, int iters, double* ops, void* stream);

/* Tuning hook for benchmarks: force the MFMA GEMM's tile configuration (0 = choose from the shape;
 * 1..28 = a fixed entry of the int4 kernel's tile table, 100 + (1..11) = of the MXFP4 kernel's; 0 resets
 * both).  Process-wide, not thread-safe. */
void pme_set_gemm_tile(int id);

/* Which kernel configuration the GEMM of a T x d_e x N layer would run under the current path and tile settings,
 * as the instantiation's name in a profiler's kernel trace (e.g. "k_gemm_mfma<256, 256, 2, 2, 128, 2, 0, 1, false>").
 * variant 0: symmetric int4, 1: asymmetric int4, 2: MXFP4.  name HOST out, at most name_len bytes with the
 * terminating zero.  Nothing is launched.  The benchmark uses it to check that stored profiler figures belong to
 * the kernel it is timing. */
pme_status pme_gemm_plan(int variant, int64_t T, int64_t d_e, int64_t N, char* name, size_t name_len);

void pme_set_path(pme_path p);
pme_path pme_get_path(void);
const char* pme_status_string(pme_status s);
int pme_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PME_H */
