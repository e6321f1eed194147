/*
 * gwq.h - C ABI of the MI355X (gfx950) library for the GWQ linear layer.
 *
 * Method: "Gradient-Aware Weight Quantization for Large Language Models" (GWQ).  Per linear
 * layer the 1 % of weights with the largest |gradient| stay FP16 and the other 99 % are
 * group-quantised to 3 or 4 bits with a per-group scale and zero point (abstract; Sec. 3.2,
 * Eq. 6-10).  The paper describes no storage format and no inference kernel; the format below
 * is this library's.
 *
 * Conventions for every call
 *   - Pointers named in a gwq_packed, and W, score, X, Y and workspaces, are DEVICE pointers
 *     owned by the caller.  The library never allocates or frees device memory.
 *   - Work is enqueued on the HIP stream passed as `stream` (a hipStream_t cast to void*;
 *     NULL = the default stream) and the call returns without waiting for it.
 *   - Arguments are validated on the host before the first HIP call; errors are returned as
 *     a gwq_status, never raised or aborted.  A failed launch returns GWQ_ERR_DEVICE.
 *   - Weights are W[N][K] row-major FP16 (N = output features, K = input features),
 *     activations X[M][K] row-major FP16, outputs Y[M][N] row-major FP16 (bfloat16 for both in
 *     gwq_linear_bf16).  No bias (Sec. 3.1 disables it).
 *
 * Packed format.  The codes of an output channel n lie in blocks of 128 consecutive k (gpr = K / 128 blocks per
 * channel), whatever the group size; scale and zero point belong to a group of `group` consecutive k of one
 * channel (Sec. 3.2, first paragraph: the group size beta, 16 in the paper; 16, 32, 64 or 128 here, spr = K / group
 * groups per channel, at most 2048).
 *   qweight  uint32 [N][gpr][wpg], wpg = 16 (4-bit) or 13 (3-bit).  A block is cut into four
 *            slots of 32 codes, slot b = k_local / 32.  Inside a word, codes at even positions
 *            sit in the low 16 bits and codes at odd positions in the high 16 bits, `bits`
 *            bits apiece, ascending.
 *            4-bit: word 4b+j (j = 0..3) holds codes 32b+8j+t (t = 0..7):
 *                   t even -> bit 4*(t/2), t odd -> bit 16+4*(t/2).
 *            3-bit: word 3b+i (i = 0..2) holds codes 32b+10i+t (t = 0..9):
 *                   t even -> bit 3*(t/2), t odd -> bit 16+3*(t/2); bits 15 and 31 are zero.
 *                   Word 12 (tail) holds code 32b+30 at bit 3b and code 32b+31 at bit 16+3b.
 *   scales   FP16 bits [N][spr]: the smallest FP16 s with s*(2^bits-1) >= max-min of the
 *            group's non-outlier weights (range widened to contain 0); 1.0 for an empty range.
 *   zeros    uint8 [N][spr]: clamp(rint(-min/s), 0, 2^bits-1).
 *   codes    clamp(rint(w/s) + z, 0, 2^bits-1), round half to even; the code under an outlier
 *            is z, so it decodes to 0 and the outlier value is added on top.
 *   row_ptr  int32 [N+1], col_idx uint16 [n_outliers] (ascending within a row), out_val FP16
 *            bits [n_outliers]: CSR of the outliers, values copied bit for bit from W.
 *   n_outliers = ceil(outlier_ppm * N * K / 1e6); the entries with the largest |score| are
 *            kept, ties going to the lowest flat index n*K + k.  |score| is ranked by its
 *            binary32 bit pattern (NaN ranks above +inf).
 */
#ifndef GWQ_H
#define GWQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GWQ_OK = 0,
    GWQ_ERR_NULL = -1,        /* a required pointer is NULL                               */
    GWQ_ERR_SHAPE = -2,       /* N, K, M out of range, K not a multiple of the group, ... */
    GWQ_ERR_UNSUPPORTED = -3, /* bits not in {3,4}, group not in {16,32,64,128}, unknown score type */
    GWQ_ERR_WORKSPACE = -4,   /* workspace missing or smaller than gwq_layout reports     */
    GWQ_ERR_DEVICE = -5       /* a HIP call failed                                        */
} gwq_status;

/* Passed as int32_t: a value outside the enumeration is answered with GWQ_ERR_UNSUPPORTED, not undefined. */
typedef enum { GWQ_SCORE_F32 = 0, GWQ_SCORE_F16 = 1 } gwq_score_dtype;

/* View of one packed layer.  Scalars are filled by the caller (n_outliers from gwq_layout). */
typedef struct {
    int32_t N, K;             /* 1 <= N, 128 <= K <= 65536, K % 128 == 0, N*K < 2^32      */
    int32_t bits;             /* 3 or 4                                                   */
    int32_t group;            /* 16, 32, 64 or 128; K / group <= 2048                     */
    uint32_t outlier_ppm;     /* 0..1000000; 10000 = 1 %                                  */
    int64_t n_outliers;       /* ceil(outlier_ppm*N*K/1e6)                                */
    uint32_t *qweight;
    uint16_t *scales;
    uint8_t *zeros;
    int32_t *row_ptr;
    uint16_t *col_idx;
    uint16_t *out_val;
    void *index;              /* optional (may be NULL): the per-layer index of gwq_linear_index, */
                              /* >= linear_index bytes, 16-byte aligned.  gwq_pack fills it when  */
                              /* set; gwq_linear then reads it for M > 16 instead of building one */
                              /* in its workspace on every call.  It must describe the layer's    */
                              /* current contents: set it to NULL for a layer packed elsewhere    */
                              /* (or fill it with gwq_linear_index).                              */
} gwq_packed;

/* Byte sizes of every buffer of a gwq_packed plus the workspaces of the two device calls. */
typedef struct {
    size_t qweight, scales, zeros, row_ptr, col_idx, out_val;
    size_t pack_workspace;    /* for gwq_pack                                             */
    size_t linear_workspace;  /* for gwq_linear with M <= M_max (0 when M_max <= 16):     */
                              /*   linear_index + linear_scratch                          */
    size_t linear_index;      /* the per-layer index of gwq_linear_index                  */
    size_t linear_scratch;    /* for gwq_linear_indexed with M <= M_max (0 when <= 16)    */
    int64_t n_outliers;
    size_t quality_workspace; /* for gwq_quality                                          */
} gwq_sizes;

/* Sizes of the buffers that hold one layer in the format above: the b-bit codes, scale and zero point of
 * Sec. 3.2 (Eq. 6, 7, 9) per group and the FP16 outliers Eq. 8 selects (pure host arithmetic, touches
 * no device; sized for the 256 compute units of gfx950).  scales, zeros, col_idx and
 * out_val are rounded up to whole 16-byte vectors plus one spare vector: gwq_linear reads them
 * with wide loads, so buffers must have these sizes and be 16-byte aligned (the padding is
 * never interpreted).
 * Errors: NULL out, shape limits above, unsupported bits/group, ppm > 1e6, M_max < 0. */
gwq_status gwq_layout(int32_t N, int32_t K, int32_t bits, int32_t group, uint32_t outlier_ppm,
                      int32_t M_max, gwq_sizes *out);

/* Encode one layer (Eq. 8 selection, then Eq. 6, 7, 9 per group, then the word layout).
 *   W_f16   device, FP16 [N][K]          score  device, [N][K] of `score_dtype`
 *   dst     host struct; its scalars describe the layer, its pointers are device buffers of
 *           the sizes gwq_layout reports; all of them are fully overwritten (dst->index too
 *           when it is not NULL)
 *   workspace device scratch of >= pack_workspace bytes, 4-byte aligned; W_f16 and score 16-byte aligned
 * The result is a function of the inputs only (bit-exact, run-to-run identical). */
gwq_status gwq_pack(const void *W_f16, const void *score, int32_t score_dtype,
                    gwq_packed *dst, void *workspace, size_t workspace_bytes, void *stream);

/* Y[M][N] = X[M][K] * (Q(W) + outliers)^T with Q(W) = s*(q-z) (Eq. 10), FP32 accumulation,
 * FP16 output.  M <= 16 takes the bandwidth-bound decode kernel, larger M the MFMA GEMM.
 *   P  host struct with device pointers   X_f16 device [M][K]   Y_f16 device [M][N]
 * X and Y must not overlap; Y is fully overwritten.  M > 16 needs `workspace`: device scratch,
 * 16-byte aligned, of the linear_workspace bytes gwq_layout reports for an M_max >= M (it is
 * rewritten by every call; concurrent calls need separate workspaces); for M <= 16 it may be
 * NULL.  The first linear_index bytes are indispensable (less: GWQ_ERR_WORKSPACE): the call
 * builds the layer's index there, unless P->index holds it already (then that part stays
 * untouched).  The rest holds FP32 partial sums when a launch also splits K, which it does where
 * rows and channels alone give too few tiles to fill the chip; with less than that the call
 * still works, without the split.
 * For M > 16, and for every M when group < 128, the weights enter the MFMA as FP16 numbers s*(q-z), with s capped
 * at the largest FP16 value for which s*(2^bits-1) is finite (4364 at 4 bits, 9352 at 3; only groups whose range
 * exceeds 65460 reach the cap, which moves such a weight by < 0.1 %); for M <= 16 and group = 128 the scale
 * multiplies FP32 sums of exact products.
 * Results are deterministic (no floating-point atomics). */
gwq_status gwq_linear(const gwq_packed *P, const void *X_f16, int32_t M, void *Y_f16,
                      void *workspace, size_t workspace_bytes, void *stream);

/* gwq_linear for bfloat16 activations (the upper half of a binary32): X_bf16 [M][K] in, Y_bf16 [M][N] out, rounded to
 * nearest even from the FP32 sums; arguments, workspace and errors as gwq_linear.  group = 128 only (else
 * GWQ_ERR_UNSUPPORTED).  Sec. 3.2 fixes the weights' format, not the activations' type; bfloat16 MFMA operands keep the
 * range of FP32 where FP16 activations overflow at 65504.  M <= 16: the MFMAs multiply x with the exact values 128 + q and
 * the scale and zero point are applied to FP32 sums.  M > 16: the weights s*(q-z) and the outliers are rounded to bfloat16
 * (8 significant bits) before the MFMA. */
gwq_status gwq_linear_bf16(const gwq_packed *P, const void *X_bf16, int32_t M, void *Y_bf16,
                           void *workspace, size_t workspace_bytes, void *stream);

/* gwq_linear in two parts, for weights that stay while activations change.  What gwq_linear writes
 * into its workspace for M > 16 depends on the packed layer alone (per channel and group: where the
 * group's outliers start, its scale and zero point), so it can be built once, when the layer is
 * loaded:
 *   gwq_linear_index   fills `index` (device, >= linear_index bytes as reported by gwq_layout,
 *                      16-byte aligned) from P;
 *   gwq_linear_indexed is gwq_linear with that index, which it only reads, so concurrent calls
 *                      may share one.  `scratch` (device, linear_scratch bytes for an M_max >= M,
 *                      16-byte aligned, one per concurrent call) is the room for the partial
 *                      sums of a K-split launch; it may be NULL or smaller: then K is not split.
 *                      For M <= 16 neither is used and both may be NULL.
 * The index is valid until P's buffers change.  Given the same scratch size as gwq_linear has
 * left after its index, the results are the same bit for bit. */
gwq_status gwq_linear_index(const gwq_packed *P, void *index, size_t index_bytes, void *stream);
gwq_status gwq_linear_indexed(const gwq_packed *P, const void *X_f16, int32_t M, void *Y_f16,
                              const void *index, size_t index_bytes, void *scratch,
                              size_t scratch_bytes, void *stream);

/* gwq_linear for callers that cannot allocate or pass a workspace (code under HIP graph capture, serving loops
 * and harnesses in which hipMalloc is off limits): the same kernels, with the scratch that M > 16 needs - the
 * layer's index when P->index is NULL, then the FP32 partial sums of a K-split launch - held in a static device
 * array of GWQ_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, for the life of the process).  The
 * call allocates and frees nothing.  Arguments and results as gwq_linear given a workspace of the
 * linear_workspace bytes gwq_layout reports for M_max = M (bit for bit).  When index (if the layer has none)
 * plus partial sums for this N and M exceed GWQ_STATIC_SCRATCH_BYTES the call returns GWQ_ERR_WORKSPACE and
 * does nothing (every shape up to 28672 x 8192 fits at any M).  All calls on a GPU share that GPU's array:
 * calls that may overlap in time on one GPU (different streams, different threads) race and must not be made;
 * calls on one stream are ordered and safe.  Nothing in the array has to start at zero. */
#define GWQ_STATIC_SCRATCH_BYTES (48u << 20)
gwq_status gwq_linear_static(const gwq_packed *P, const void *X_f16, int32_t M, void *Y_f16, void *stream);

/* Several layers in one decode launch (M <= 16): Y_f16[i] = gwq_linear(P[i], X_f16[i]) for
 * i < count <= GWQ_MAX_BATCH.  For layers with no data dependence between them, such as the q, k
 * and v or the gate and up projections of a decoder layer (which may share one X): at decode sizes a
 * launch is dominated by latency rather than bandwidth, and one launch over more bytes hides it
 * (the paper's efficiency table, Sec. 4.2, measures whole-model decode).  All layers must have the same
 * `bits`; N and K may differ (layers of equal K share a launch, so a batch with two values of K takes two).
 * P, X_f16 and Y_f16 are HOST arrays of `count` pointers (to host structs / device buffers); they are
 * read before the call returns.  Same rules as gwq_linear. */
#define GWQ_MAX_BATCH 8
gwq_status gwq_linear_batch(int32_t count, const gwq_packed *const *P, const void *const *X_f16,
                            int32_t M, void *const *Y_f16, void *stream);

/* Figures of merit of a packed layer against the weights W it was packed from (Sec. 3.1).  With W_Q
 * the decoded layer - s*(q-z) (Eq. 10) where a weight was quantised, the stored FP16 value where it was
 * kept - and D = W - W_Q:
 *   out[0] = sum D^2          the squared error the quantiser minimises (Eq. 4)
 *   out[1] = sum score * D    g^T (W - W_Q): the first-order change of the loss (Eq. 3 and 5) when
 *                             `score` is the gradient the outliers were ranked by
 *   out[2] = max |D|
 *   W_f16 device [N][K], score device [N][K] of `score_dtype` (both 16-byte aligned), out_f64 device, 3 doubles,
 *   8-byte aligned;
 *   workspace device, >= quality_workspace bytes as gwq_layout reports, 8-byte aligned.
 * Every D is exact (fp64 from FP16 operands); the sums are fp64 in a fixed order, so the results are
 * identical from run to run.  Inputs are expected to be finite. */
gwq_status gwq_quality(const gwq_packed *P, const void *W_f16, const void *score, int32_t score_dtype,
                       double *out_f64, void *workspace, size_t workspace_bytes, void *stream);

/* The score that gwq_pack ranks, for one linear layer (Sec. 3.1, Eq. 2: the gradient of the loss with
 * respect to the weights).  For Y = X W^T without bias the chain rule gives it from the gradient dY of the
 * loss with respect to Y:
 *   g[n][k] = sum over m of dY[m][n] * X[m][k]
 *   score[n][k] = beta * score[n][k] + alpha * g[n][k]
 * so the mean over calibration samples (Sec. 4.3, ablation on the number of calibration samples) is one call per sample or batch of samples with
 * alpha = 1 / samples, beta = 0 on the first call (score is then not read: it may be uninitialised)
 * and 1 afterwards.
 *   dY_f16  device [M][N] row-major FP16; 16-byte aligned when N is a multiple of 8, else 2-byte
 *   X_f16   device [M][K] row-major FP16, 16-byte aligned; K a multiple of 128, <= 65536 (as gwq_pack)
 *   score_f32 device [N][K] row-major FP32, 4-byte aligned: what gwq_pack takes as GWQ_SCORE_F32
 *   M >= 1, 1 <= N <= 2^24
 * Products are exact, sums FP32 (MFMA); deterministic.  No workspace. */
gwq_status gwq_score(const void *dY_f16, const void *X_f16, int32_t M, int32_t N, int32_t K, float alpha,
                     float beta, float *score_f32, void *stream);

/* The gated pair of a decoder layer's MLP in decode (M <= 16):
 *   H[m][n] = silu(G[m][n]) * U[m][n],   G = gwq_linear(P_gate, X),  U = gwq_linear(P_up, X),  silu(x) = x / (1 + e^-x)
 * What the efficiency table (Sec. 4.2) times is whole-model generation, where every decoder layer runs this pair
 * and then the down projection on H; at decode sizes a launch is bound by latency, so for M <= 4 both products
 * and the gate are one launch (the FP32 sums of the gate product never leave the block) and G and U are never
 * written.  For 5 <= M <= 16 (and rows too long for that kernel) the two products go to `workspace` (device,
 * >= 4*M*N bytes, 16-byte aligned; may be NULL for M <= 4 with K <= 16384) and a third launch combines them.
 * P_gate and P_up must agree in N, K and bits.  H_f16 device [M][N], fully overwritten.  For M <= 4 H is
 * computed from the FP32 sums; otherwise from the FP16-rounded products.  Other rules as gwq_linear. */
gwq_status gwq_linear_gate_up(const gwq_packed *P_gate, const gwq_packed *P_up, const void *X_f16, int32_t M, void *H_f16,
                              void *workspace, size_t workspace_bytes, void *stream);

/* Which kernel gwq_linear (count = 1) or gwq_linear_batch (layers of one K) would launch for these layers and M:
 * kernel name with its template arguments, grid, block, LDS bytes, written as text (NUL-terminated, truncated
 * to text_bytes).  Pure host call: reads the structs' scalars (and the tuning hooks), launches nothing, so a
 * benchmark can label its numbers with the kernel that actually ran.  with_scratch: for M > 16, whether the
 * call has the scratch for a K-split launch.  Errors as gwq_linear_batch; M > 16 needs count = 1. */
gwq_status gwq_linear_plan(int32_t count, const gwq_packed *const *P, int32_t M, int32_t with_scratch, char *text,
                           size_t text_bytes);

/* Measurement probes for the ceilings the kernels are compared with (no part of the method: the paper gives no
 * kernel and no hardware numbers; the benchmark runs these beside the real kernels, launched the same way).
 *   gwq_probe_stream  one plain streaming read of `bytes` (a multiple of 16, 16-byte aligned) of device memory:
 *                     what moving the same bytes takes with no arithmetic at all;
 *   gwq_probe_mfma    `blocks` blocks of four waves, each wave issuing 8 * iters v_mfma_f32_32x32x16_f16 out of
 *                     registers: 2 * 32*32*16 * 8 * iters * 4 * blocks floating-point operations.
 * sink: 4 bytes of device memory (practically never written). */
gwq_status gwq_probe_stream(const void *src, size_t bytes, void *sink, void *stream);
gwq_status gwq_probe_mfma(int32_t blocks, int32_t iters, void *sink, void *stream);

/* Launch-shape overrides for measurement sweeps; value 0 restores the built-in heuristic.  The values are
 * process-wide (atomic, read once per call by every thread's calls): a hook for benchmarks and tests, not a
 * per-call option.
 * Keys: "decode_waves" (upper bound, 1..16, on the waves per block of the decode kernel for M <= 8:
 * it picks 4, 8 or 16 groups per wave accordingly; the kernels for larger M size themselves),
 * "decode_stream" (1: never the streaming decode kernel; 2: also for M <= 4, wherever K <= 4096 lets it
 * run; by default it takes the launches of 5 <= M <= 16 there that the kernel for M <= 8 does not, with two or more tiles per block), "decode_tiles" (16-channel tiles per block of the streaming
 * kernel, 1..4096), "decode_lean_rows" (1..8: the largest M handled by the kernel that keeps all of X[M][K] in LDS,
 * where it fits), "decode_pairs" (that kernel with two neighbouring 16-channel tiles per block, which share one copy of X
 * in LDS, for 5 <= M <= 8: 1 never, 2 wherever it fits; by default where the launch has at least four tiles per compute
 * unit), "pack_full_passes" (1: gwq_pack finds the threshold and the per-row counts by passes over all
 * scores even where the short list of candidate keys would do), "gemm_rows" (rows of Y per block of the GEMM: 32, 64, 128 or 256; by default 256 beyond
 * M = 512 and below that the shape a cost model of the launch expects to be fastest).  Unknown keys or
 * out-of-range values return GWQ_ERR_UNSUPPORTED. */
gwq_status gwq_tuning_set(const char *key, int32_t value);

const char *gwq_status_string(gwq_status status);
const char *gwq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GWQ_H */
