/*
 * sfb.h -- C ABI of the MI355X (gfx950) library for the data-parallel hot path of
 * Sufficient Factor Broadcasting (SFB).
 *
 * One bulk-synchronous SFB iteration for a matrix-parametrised model
 *     min_W (1/N) sum_i f_i(W a_i) + h(W),   W in R^{J x D}          (Section 2, problem (P))
 * on P simulated workers that each hold B samples of the minibatch and an identical
 * replica of W (Section 3; replicas are equal under BSP, Section 4.1):
 *
 *   factors      u_i = d f_i(W a_i) / d (W a_i),  v_i = a_i            (Section 2.1, proximal SGD)
 *   exchange     worker p's B pairs land in rows [p*B, (p+1)*B) of the concatenated
 *                buffers U[N][J], V[N][D], N = P*B: what every worker holds once all
 *                broadcasts have arrived                                (Section 3)
 *   reconstruct  dW = sum_p (1/B) sum_i u_{p,i} v_{p,i}^T               (Section 3, sum over
 *                workers; mini-batch paragraph, mean over a worker's K = B samples)
 *   apply        W <- W - eta * dW; prox is the identity (h = 0)        (Section 2.1)
 *
 * Conventions that hold for every entry point:
 *   - Every matrix is ROW-MAJOR with an explicit leading dimension counted in ELEMENTS.
 *   - Every data pointer (W, features, labels, U, V, loss, workspace) is DEVICE memory owned
 *     by the caller.  The library allocates and frees no device memory and keeps no data
 *     pointer after a call returns, except the workspace registered with sfb_set_workspace.
 *     The only HOST data pointer is the `active` mask.  Struct arguments (sfb_batch) live on
 *     the host and are read during the call only.
 *   - Calls enqueue kernels on the context's HIP stream and return without synchronising.
 *     A launch failure is returned at once as SFB_EHIP; a fault during execution surfaces
 *     at sfb_sync or at the next call.
 *   - Errors are reported by the integer return value only.  If validation fails no kernel
 *     is launched and no output is touched.
 *   - Any alignment and any leading dimension >= the row length is accepted; pointers that
 *     are 16-byte aligned with leading dimensions that are multiples of 4 elements (8 for
 *     bf16) take the vectorised paths.
 *   - Class ids in `y` outside [0, J) are not detected on the device (the one-hot term is
 *     then simply absent); callers validate labels.
 *   - A context is not thread-safe; distinct contexts are independent.
 */
#ifndef SFB_H
#define SFB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SFB_API __attribute__((visibility("default")))

typedef struct sfb_ctx sfb_ctx; /* opaque, host-side dispatch state only */

/* Loss families (f_i of problem (P), Section 2). */
typedef enum {
    SFB_MLR = 0,   /* multiclass logistic: f = logsumexp(z) - z_y; u = softmax(z) - e_y          */
    SFB_DML = 1,   /* distance metric learning: a = x - y (pair difference), z = W a;
                      similar pair f = |z|^2, u = 2z; dissimilar f = max(0, 1 - |z|^2),
                      u = -2z if |z|^2 < 1 else 0 (Section 2, DML paragraph)                     */
    SFB_L2SVM = 2  /* one-vs-rest squared hinge, t_j = +1 if j == y else -1:
                      f = sum_j max(0, 1 - t_j z_j)^2, u_j = -2 t_j max(0, 1 - t_j z_j);
                      features given as CSR                                                      */
} sfb_model;

/* Storage type of the features and of V.  W, U, loss and the workspace are always fp32. */
typedef enum { SFB_F32 = 0, SFB_BF16 = 1 } sfb_dtype;

typedef enum {
    SFB_OK = 0,
    SFB_EINVAL = -1,       /* null pointer, non-positive size, non-finite eta or scale      */
    SFB_ESHAPE = -2,       /* leading dimension shorter than the row, nnz < 0, p out of range */
    SFB_EDTYPE = -3,       /* unknown dtype                                                  */
    SFB_EWORKSPACE = -5,   /* workspace missing or smaller than sfb_workspace_bytes          */
    SFB_EUNSUPPORTED = -6, /* (model, dtype) combination or size the kernels do not cover    */
    SFB_EHIP = -7,         /* a HIP call failed; see sfb_last_hip_error                      */
    SFB_ESCRATCH = -8      /* sfb_step_noalloc: the context needs more scratch than
                              SFB_NOALLOC_SCRATCH_BYTES                                      */
} sfb_status;

/*
 * One minibatch, already laid out as P contiguous partitions of B samples (worker p's draw
 * is rows [p*B, (p+1)*B)).  Host struct of DEVICE pointers.
 *   MLR:    a = features [N][lda] in the context's dtype; a2 = csr_* = NULL.
 *   DML:    a = first point of each pair, a2 = second point, both [N][lda] (fp32 only).
 *   L2SVM:  a = a2 = NULL; CSR with N rows and D columns: csr_rowptr [N+1] (int32, first
 *           entry is this batch's offset into csr_col/csr_val, normally 0), csr_col [nnz]
 *           in [0, D), csr_val [nnz] fp32, nnz = total stored entries.  Columns may appear
 *           in any order; a column repeated inside a row counts as the sum of its values
 *           (in the scores and in the dense row v_i alike).
 */
typedef struct sfb_batch {
    const void *a;
    const void *a2;
    int64_t lda;
    const int32_t *csr_rowptr;
    const int32_t *csr_col;
    const float *csr_val;
    int64_t nnz;
} sfb_batch;

/*
 * Create a context for model `m`, W of J x D, P workers x B samples, feature storage type
 * `input_dtype`, enqueueing on `hip_stream` (a hipStream_t; NULL = the default stream).
 * Mirrors the paper's constructor sfb_app(J, D, staleness) (Section 4.2) without staleness:
 * only the bulk-synchronous mode exists here.
 */
SFB_API sfb_status sfb_create(sfb_ctx **out, sfb_model m, int64_t J, int64_t D, int32_t P, int32_t B,
                      sfb_dtype input_dtype, void *hip_stream);
SFB_API void sfb_destroy(sfb_ctx *ctx);

/* Bytes of device workspace the context needs: the scores Z[N][J] as split-K partial sums,
 * plus, for bf16 contexts, the transposed bf16 copies of the factors that the
 * reconstruction multiplies (so sfb_reconstruct_apply needs the workspace too).  fp32 contexts
 * whose J is not a multiple of 4, D not one of 128 or P*B not one of 32 also count room for padded
 * fp32 copies of U and V (rows of J rounded up to 4 and D rounded up to 128 floats, P*B rounded up
 * to 32 rows; the same bytes as the partial scores, which are dead by then): with it registered
 * their reconstruction runs the same matrix-core kernels as whole shapes, whatever the alignment
 * of U, V and W, without it the slower element-by-element kernel (same results to rounding).  A
 * call with a dead worker (`active`) likewise takes a masked copy of U in the partial scores' bytes, and
 * shapes of a few 64 x 64 tiles of W with thousands of factor pairs count planes of partial sums (the
 * pairs are then cut into slices over workgroups and added in a fixed order).  The
 * caller allocates at least that many bytes, 256-byte aligned, and registers them; the library
 * uses the buffer until it is replaced or the ctx destroyed. */
SFB_API sfb_status sfb_workspace_bytes(const sfb_ctx *ctx, size_t *bytes);
SFB_API sfb_status sfb_set_workspace(sfb_ctx *ctx, void *dev, size_t bytes);

/*
 * Factors of all N = P*B samples, every sample differentiated at the same W
 * (Section 2.1; Section 4.2: write_u / write_v / commit of every worker).
 *   W     [J][ldw] fp32, read only.
 *   y     [N] int32: class id (MLR, L2SVM) or 1 = similar / 0 = dissimilar (DML).
 *   U     [N][ldu] fp32 out: u_i, unscaled (MLR rows sum to 0).
 *   V     [N][ldv] out, context dtype: v_i = a_i (DML: x_i - y_i; L2SVM: the dense row).
 *   loss  [N] fp32 out or NULL: f_i(W a_i).
 */
SFB_API sfb_status sfb_compute_factors(sfb_ctx *ctx, const float *W, int64_t ldw, const sfb_batch *batch,
                               const int32_t *y, float *U, int64_t ldu, void *V, int64_t ldv,
                               float *loss);

/*
 * One worker's share: `batch_p` and `y_p` hold that worker's B samples only (B rows; CSR with
 * B rows); the call writes rows [p*B, (p+1)*B) of U, V (and loss) and nothing else -- one
 * worker's commit() into slot p of everybody's receive buffer (Section 4.2, Section 3).
 * U, V, loss are the base pointers of the full N-row buffers.
 */
SFB_API sfb_status sfb_compute_factors_worker(sfb_ctx *ctx, const float *W, int64_t ldw,
                                      const sfb_batch *batch_p, const int32_t *y_p, int32_t p,
                                      float *U, int64_t ldu, void *V, int64_t ldv, float *loss);

/*
 * W <- W - eta * scale * sum over live workers p, samples i of u_{p,i} v_{p,i}^T, in place
 * (Section 3 reconstruction fused with the Section 2.1 update).  scale = 1/B gives the
 * mini-batch mean of Section 3; scale = 1 the plain sum.  `active` is a HOST array of P
 * bytes (0 = that worker's factors never arrived, cf. Section 4.4) or NULL for all live;
 * with a mask P must be <= 64.  U and V are not modified.
 */
SFB_API sfb_status sfb_reconstruct_apply(sfb_ctx *ctx, float *W, int64_t ldw, const float *U, int64_t ldu,
                                 const void *V, int64_t ldv, float eta, float scale,
                                 const uint8_t *active);

/*
 * One worker's factors only: W <- W - eta * scale * sum_i u_{p,i} v_{p,i}^T over rows
 * [p*B, (p+1)*B) of U and V (base pointers of the full N-row buffers) -- what a replica does
 * when the sufficient factors of worker p arrive (Section 3; Section 4.1: under the
 * asynchronous and stale-synchronous models arrivals are applied one sender at a time).
 * Costs a contraction over B rows, not over N.
 */
SFB_API sfb_status sfb_reconstruct_apply_worker(sfb_ctx *ctx, float *W, int64_t ldw, const float *U,
                                        int64_t ldu, const void *V, int64_t ldv, int32_t p, float eta,
                                        float scale);

/* sfb_compute_factors followed by sfb_reconstruct_apply with scale = 1/B: one full BSP
 * iteration.  U, V (and loss) hold the step's factors afterwards. */
SFB_API sfb_status sfb_step(sfb_ctx *ctx, float *W, int64_t ldw, const sfb_batch *batch, const int32_t *y,
                    float *U, int64_t ldu, void *V, int64_t ldv, float *loss, float eta,
                    const uint8_t *active);

/*
 * The same iterations regrouped so that W crosses memory once per iteration instead of three
 * times: apply the pending factors (U, V hold those of iteration t: the update of Section 2.1 with the
 * reconstruction of Section 3, scale 1/B), then compute the factors of iteration t+1 at the W just
 * produced (Section 2.1: every iteration differentiates at the current W), leaving them in U, V
 * (and loss) as the new pending factors.  A run is
 *     sfb_compute_factors(W, batch_0) ; sfb_step_pipelined(W, batch_1) ; ... ; sfb_step_pipelined(W, batch_T-1) ;
 *     sfb_reconstruct_apply(W, U, V, eta, 1/B)
 * and gives what T calls of sfb_step give.  For bf16 contexts whose shape the fused kernel covers
 * (P*B in {128, 256, 512}, D a multiple of 32, J*ldw < 2^31, 16-byte aligned operands) the update and
 * the next scores run in ONE kernel that reads and writes every tile of W once; otherwise the call runs
 * sfb_reconstruct_apply and sfb_compute_factors one after the other (same results as sfb_step).
 * `active` masks the workers of the PENDING factors.  The next batch's features must not overlap V
 * (V is read as v_t and overwritten with the next features piece by piece).  Needs the registered
 * workspace (query sfb_workspace_bytes).  Errors as sfb_step; nothing is launched if an argument is refused.
 * sfb_pipeline_info: whether the fused kernel is what the context would run (0 / 1), its grid and
 * its number of column slices (0 when not fused); any pointer may be NULL.
 */
SFB_API sfb_status sfb_step_pipelined(sfb_ctx *ctx, float *W, int64_t ldw, float *U, int64_t ldu, void *V,
                                      int64_t ldv, const sfb_batch *next_batch, const int32_t *next_y,
                                      float *loss, float eta, const uint8_t *active);
SFB_API sfb_status sfb_pipeline_info(const sfb_ctx *ctx, int32_t *fused, int32_t *grid, int32_t *slices);

/*
 * sfb_step for callers that cannot allocate or register device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * same results as sfb_step, bit for bit, but the scratch the kernels need (split-K partial scores,
 * padded factor copies of ragged fp32 shapes, packed bf16 factors) is a fixed array of SFB_NOALLOC_SCRATCH_BYTES of device memory inside the library, one copy per
 * GPU, instead of the workspace registered with sfb_set_workspace (which this call neither needs
 * nor touches).  The call allocates and frees nothing, on the host or on the device.
 *   - SFB_ESCRATCH (nothing launched) if sfb_workspace_bytes(ctx) exceeds SFB_NOALLOC_SCRATCH_BYTES;
 *     of the benchmark shapes every one but the 10000 x 21504 bf16 one fits.
 *   - The context must have been created with the GPU current that the call runs on (sfb_create
 *     resolves the array's address for that GPU).
 *   - All calls on one GPU share that GPU's array, from whatever context or stream: calls that may
 *     overlap in time race on it.  Serialise them (one stream, or events between streams).
 *     Nothing needs clearing between calls: a step writes every scratch byte before it reads it.
 */
#define SFB_NOALLOC_SCRATCH_BYTES ((size_t)16 << 20)
SFB_API sfb_status sfb_step_noalloc(sfb_ctx *ctx, float *W, int64_t ldw, const sfb_batch *batch,
                                    const int32_t *y, float *U, int64_t ldu, void *V, int64_t ldv,
                                    float *loss, float eta, const uint8_t *active);

/*
 * SFB driven by stochastic dual coordinate ascent (Section 2.1, "Stochastic DCA") for the
 * l2-regularised multiclass logistic regression, h(W) = lam/2 ||W||_F^2 (SFB_MLR contexts only).
 * Every data sample i owns a dual vector u_i in R^J; the primal matrix is tied to them by
 * W = grad h*(Z) = Z / lam with Z = (1/n_data) sum_i u_i a_i^T.  One iteration picks P*B
 * DISTINCT data samples (batch row r is data sample sample[r]); for each of them, with the
 * scores z = W a at the iteration's start,
 *     delta u_i = s * (u_i - (e_y - softmax(z))),     u_i <- u_i - delta u_i,
 * (the step of proximal SDCA: a fraction s in (0, 1] of the way to the dual vector that is
 * optimal for the current scores), and the pair (delta u_i, a_i) is the sufficient factor:
 *     W <- W - 1/(lam n_data) * sum_i delta u_i a_i^T
 * which is sfb_reconstruct_apply with eta = 1 and scale = 1/(lam n_data).
 * Start from dual = 0 and W = 0 (or any pair that satisfies the tie above).
 *   dual    DEVICE [n_data][ld_dual] fp32, updated in place at the picked rows.
 *   sample  DEVICE [N] int32 in [0, n_data), distinct within the call (not checked: two rows
 *           naming one sample race on its dual vector).
 *   conj    DEVICE [n_data] fp32 or NULL: entry sample[r] receives f*(-u) = sum_j p_j log p_j,
 *           p = e_y - u, of the updated dual vector (the sample's term of the dual objective).
 */
typedef struct sfb_sdca {
    float *dual;
    int64_t ld_dual;
    int64_t n_data;
    const int32_t *sample;
    float *conj;
    float lam;
    float s;
} sfb_sdca;
/* Factors of one SDCA iteration: U [N][ldu] = delta u_i, V = a_i, loss [N] = f_i(W a_i) or NULL;
 * the dual vectors of the picked samples are updated.  W is read only.
 * SFB_EINVAL: null dual / sample, n_data < 1, lam <= 0 or s outside (0, 1] or not finite;
 * SFB_ESHAPE: ld_dual < J; SFB_EUNSUPPORTED: the context's model is not SFB_MLR. */
SFB_API sfb_status sfb_sdca_compute_factors(sfb_ctx *ctx, const float *W, int64_t ldw, const sfb_batch *batch,
                                    const int32_t *y, const sfb_sdca *sdca, float *U, int64_t ldu,
                                    void *V, int64_t ldv, float *loss);
/* sfb_sdca_compute_factors followed by the reconstruction above: one full SDCA iteration. */
SFB_API sfb_status sfb_sdca_step(sfb_ctx *ctx, float *W, int64_t ldw, const sfb_batch *batch, const int32_t *y,
                         const sfb_sdca *sdca, float *U, int64_t ldu, void *V, int64_t ldv, float *loss);

/*
 * The proximal step of proximal SGD (Section 2.1): W <- prox_{eta h}(W), in place, to be called
 * after sfb_step / sfb_reconstruct_apply when h is not 0.  Regularisers of Section 2 with a
 * closed form per entry or per column (the trace norm is not covered):
 *   SFB_PROX_NONE         h = 0: nothing is launched
 *   SFB_PROX_L2SQ         h = param/2 ||W||_F^2:        W <- W / (1 + eta param)
 *   SFB_PROX_L1           h = param ||W||_1:            W <- sign(w) max(|w| - eta param, 0)
 *   SFB_PROX_COLUMN_BALL  h = indicator of ||W_k||_2 <= param for every column k (sparse coding:
 *                         dictionary columns inside the ball); W_k <- W_k min(1, param / ||W_k||_2),
 *                         eta is ignored; needs the registered workspace.
 * SFB_EINVAL: null W, unknown kind, eta or param negative or not finite, radius 0;
 * SFB_ESHAPE: ldw < D; SFB_EWORKSPACE: column ball without a registered workspace.
 * Timed under family 4 (for the column ball: the pass that forms the column norms).
 */
typedef enum {
    SFB_PROX_NONE = 0,
    SFB_PROX_L2SQ = 1,
    SFB_PROX_L1 = 2,
    SFB_PROX_COLUMN_BALL = 3
} sfb_prox_kind;
SFB_API sfb_status sfb_prox(sfb_ctx *ctx, float *W, int64_t ldw, sfb_prox_kind kind, float eta, float param);
/* One proximal-SGD iteration (Section 2.1): sfb_reconstruct_apply / sfb_step followed by
 * prox_{eta h}.  The entrywise kinds (squared l2, l1) are applied to every updated entry of W
 * before the reconstruction stores it -- same result as the separate call, bit for bit, without
 * its pass over W; the column projection runs as its own kernels after the update.
 * Errors: those of the two calls; nothing is launched if any argument is refused. */
SFB_API sfb_status sfb_reconstruct_apply_prox(sfb_ctx *ctx, float *W, int64_t ldw, const float *U, int64_t ldu,
                                      const void *V, int64_t ldv, float eta, float scale,
                                      const uint8_t *active, sfb_prox_kind kind, float param);
SFB_API sfb_status sfb_step_prox(sfb_ctx *ctx, float *W, int64_t ldw, const sfb_batch *batch, const int32_t *y,
                         float *U, int64_t ldu, void *V, int64_t ldv, float *loss, float eta,
                         const uint8_t *active, sfb_prox_kind kind, float param);

/* What the context was created with; any pointer may be NULL. */
SFB_API sfb_status sfb_shape(const sfb_ctx *ctx, int64_t *J, int64_t *D, int32_t *P, int32_t *B,
                     int32_t *input_dtype);

/* The scale sfb_step uses: 1/B as fp32, the mean over a worker's K = B samples (Section 3,
 * mini-batch paragraph).  Callers of sfb_reconstruct_apply that want the same update as
 * sfb_step pass this value. */
SFB_API sfb_status sfb_default_scale(const sfb_ctx *ctx, float *scale);

/* hipStreamSynchronize on the context's stream; SFB_EHIP if the stream reports an error. */
SFB_API sfb_status sfb_sync(sfb_ctx *ctx);

/* Static description of a status code. */
SFB_API const char *sfb_strerror(sfb_status s);
/* Last hipError_t seen by this context (0 = hipSuccess). */
SFB_API int sfb_last_hip_error(const sfb_ctx *ctx);

/*
 * Read back the launch plan chosen at creation (for benches and tests): number of split-K
 * slices of the score contraction, and the elapsed-time bookkeeping switch.  When timing is
 * enabled the main kernel of every family is launched with a pair of HIP events attached to its
 * own dispatch (start and stop timestamps of that kernel, nothing else in between; do not
 * enable it while the stream is being captured into a graph); sfb_kernel_time_ms synchronises
 * and returns the accumulated milliseconds and launch count of kernel family `which`
 * (0 = scores, 1 = factor u, 2 = reconstruct-apply: the contraction, without the bf16 path's
 * operand-packing kernel, 3 = CSR densify / stream copy, 4 = proximal step, 5 = the one-pass update +
 * next scores kernel of sfb_step_pipelined, without its packing kernel) since the last reset.
 */
SFB_API sfb_status sfb_plan_info(const sfb_ctx *ctx, int32_t *fwd_split_k, int32_t *fwd_grid,
                         int32_t *recon_grid);
/* Tuning override of the launch plan: forward tile (bm, bn in {64, 128}), split-K slices,
 * reconstruct tile variant (rows x columns of W / wavefronts: 0: 128x128/4, 1: 64x128/2,
 * 2: 32x128/1, 3: 256x128/4, 4: 128x128/8, 5: 64x128/4, 6: 128x128/4 with 64-row wavefronts;
 * 4-6 split each stage's factor pairs between two wavefronts per row group; 7: 128x128/4,
 * 8: 64x128/2 staged by LDS-DMA where the shape allows, else as 0, 1; 9: 64x64/4, one 32x32 block per
 * wavefront, LDS-DMA, else as 8; 10: as 7 with 16-pair stages and two workgroups per compute unit;
 * 11: (96, 128 or 160)x64/8, the eight wavefronts split the two column blocks, every stage's factor
 * pairs and the stages themselves, LDS-DMA, for J whose 32-row blocks divide into tiles of 3 to 5, else as 9;
 * 12: 128x128/8, two wavefronts per 32-row strip that take the stages in turn, LDS-DMA, else as 7).
 * fp32 contexts that keep padded factor copies (see sfb_workspace_bytes) run 9, 11 or 12 on the copies:
 * 8 stands for 9 there, 7 and 10 for 12, 11 outside its range of J for 9; 0-6 take the factors as they are.
 * fwd_dma: bit 0 = stage the score contraction's tiles by LDS-DMA where the shape allows (else
 * always through registers); bit 1 = L2SVM scores always by the dense contraction on the densified rows,
 * bit 5 = always from the CSR entries where that kernel can take them (four rows of W in LDS: D <= 10240)
 * (neither: whichever a fitted cost comparison on N, J, D and nnz expects to be faster); bit 2 = fp32 scores on the bf16 matrix cores, every fp32 operand split
 * exactly into three bf16 terms and every product taken as its six leading term products (error
 * at the level of one fp32 rounding; full batch and 16-byte aligned rows only, else ignored);
 * bit 3 = the same for the fp32 reconstruction (J, D multiples of 4, N a multiple of 32, no dead
 * workers, else ignored); bit 4 = sfb_step_pipelined always runs its two separate passes; < 0 = keep.  A value <= 0 (variant < 0) keeps the current choice.
 * The workspace requirement may grow: query sfb_workspace_bytes again.  SFB_EINVAL for a value outside the table. */
SFB_API sfb_status sfb_set_plan(sfb_ctx *ctx, int32_t fwd_bm, int32_t fwd_bn, int32_t fwd_split_k,
                                int32_t recon_variant, int32_t fwd_dma);
/* Measurement aid, not part of the method: dst[0..bytes) = src[0..bytes) with a plain streaming
 * kernel on the context's stream (both DEVICE, 16-byte aligned, bytes a multiple of 16; else
 * SFB_EINVAL).  Gives the achievable copy bandwidth of the part and a known-size kernel for
 * calibrating hardware traffic counters.  Timed under family 3. */
SFB_API sfb_status sfb_stream_copy(sfb_ctx *ctx, void *dst, const void *src, size_t bytes);
/*
 * Measurement aids, not part of the method: one launch that does only the memory traffic or only
 * the matrix-core work of one of the path's kernels, in that kernel's access shape, on the
 * context's stream; timed under family 3.  They give the floors the kernels are compared with.
 *   SFB_PROBE_W_STREAM  reads W [J][ldw] once the way the bf16 score pass does (blocks of 256 rows
 *                       walked along a slice of D, 128 bytes per row and step); param = how many
 *                       workgroups read every block (1, or 2 = the score pass at N = 512).  W must
 *                       be 16-byte aligned with ldw % 4 == 0 and D % 32 == 0 (else SFB_EUNSUPPORTED).
 *   SFB_PROBE_W_RMW     W += 0 in the tile and lane mapping of the bf16 reconstruction's update
 *                       (256 x 128 tiles, accumulator layout); W keeps its values; param ignored.
 *   SFB_PROBE_MFMA_F32  register-resident loop of v_mfma_f32_32x32x2_f32 on every compute unit, param = 1
 *   SFB_PROBE_MFMA_BF16 or 2 wavefronts per SIMD; 256 * 4 * param wavefronts run SFB_PROBE_MFMA_ITERS * 16
 *                       instructions each (4096 resp. 32768 flop per instruction); W is ignored.
 *   SFB_PROBE_EMPTY     an empty kernel of 256 workgroups: what a dispatch costs (W and param ignored).
 *   SFB_PROBE_FUSED_TRAFFIC  the memory operations of sfb_step_pipelined's one-pass kernel and nothing else, in
 *                       its grid: per tile of 128 rows x 32 columns the copies of the packed v^T and
 *                       feature tiles and of the W tile into LDS and the stores of the W tile (the values
 *                       just read: W keeps its bits); no matrix work, no barriers.  For contexts whose
 *                       sfb_pipeline_info says fused, W 16-byte aligned with ldw % 4 == 0 (else
 *                       SFB_EUNSUPPORTED); needs the whole registered workspace (its packed-operand areas
 *                       are read, whatever they hold); param ignored.
 * Needs a registered workspace (64 floats of it are scribbled on).  SFB_EINVAL: null W where one is
 * needed, param outside its range, unknown kind.
 */
typedef enum {
    SFB_PROBE_W_STREAM = 0,
    SFB_PROBE_W_RMW = 1,
    SFB_PROBE_MFMA_F32 = 2,
    SFB_PROBE_MFMA_BF16 = 3,
    SFB_PROBE_EMPTY = 4,
    SFB_PROBE_FUSED_TRAFFIC = 5
} sfb_probe_kind;
#define SFB_PROBE_MFMA_ITERS 4000
SFB_API sfb_status sfb_probe(sfb_ctx *ctx, sfb_probe_kind kind, float *W, int64_t ldw, int32_t param);
SFB_API sfb_status sfb_enable_timing(sfb_ctx *ctx, int enable);
SFB_API sfb_status sfb_kernel_time_ms(sfb_ctx *ctx, int which, double *ms, int64_t *launches);
SFB_API sfb_status sfb_reset_timing(sfb_ctx *ctx);

/*
 * Stale-synchronous SFB (Section 4.1, "SSP-SFB"; local update rule of Section 5) simulated on
 * one device: P replicas of W, one per worker, that the caller owns and initialises to the
 * same W^0.  The caller drives the schedule (who computes, what arrives where and when);
 * this object keeps the clocks, enforces the two rules and runs the kernels:
 *   t_p        iterations worker p has completed;
 *   tau[p][q]  how many of worker q's factor sets replica p has applied (tau[p][p] = t_p: a
 *              worker applies its own factors at once);
 *   staleness  worker p may start its next iteration only while t_p - tau[p][q] <= staleness
 *              for every q; otherwise it pauses (staleness 0 = bulk-synchronous);
 *   no fast-forward  tau[p][q] <= t_p: a replica never applies more of q's iterations than it
 *              has completed itself (the condition tau_p^q(c) <= c - 1 of Section 5).
 * Worker q's factors of iteration t live in rows [q*B, (q+1)*B) of slot t % ring_slots of the
 * ring buffers until every replica has applied them; ring_slots >= 2*staleness + 2 (the two
 * rules bound t_q - tau[p][q] by 2*staleness + 2: q is at most staleness + 1 ahead of p, and p
 * at most staleness + 1 ahead of what it has applied of q).  Each set is applied with the eta of the
 * iteration that produced it and scale 1/B.
 * If a kernel launch fails in the middle of an event (SFB_EHIP), the replicas and the clocks no
 * longer describe the same state: that status is returned by every later event of the simulator.
 *   W_replicas  HOST array of P DEVICE pointers, each [J][ldw] fp32.
 *   U_ring      DEVICE [ring_slots][N][ldu] fp32;  V_ring  DEVICE [ring_slots][N][ldv] in the
 *               context's dtype.  The ctx must outlive the simulator; its workspace must be set.
 */
typedef struct sfb_ssp sfb_ssp;
SFB_API sfb_status sfb_ssp_create(sfb_ssp **out, sfb_ctx *ctx, int32_t staleness, float *const *W_replicas,
                          int64_t ldw, float *U_ring, int64_t ldu, void *V_ring, int64_t ldv,
                          int32_t ring_slots);
SFB_API void sfb_ssp_destroy(sfb_ssp *ssp);
/* Worker p's next iteration on its own B samples (as in sfb_compute_factors_worker), at its
 * own replica: factors into the ring, own update applied, t_p += 1.  If the staleness rule
 * forbids it, *blocked = 1 and nothing else happens (SFB_OK); if the ring slot of this
 * iteration still holds a set that one of p's receivers has not applied (the send queue is
 * full: cannot happen under full broadcast with ring_slots >= 2*staleness + 2), *blocked = 2
 * and nothing else happens; else *blocked = 0.
 * loss: base of a DEVICE [N] fp32 array of which rows [p*B, (p+1)*B) are written, or NULL. */
SFB_API sfb_status sfb_ssp_worker_step(sfb_ssp *ssp, int32_t p, const sfb_batch *batch_p, const int32_t *y_p,
                               float eta, float *loss, int32_t *blocked);
/* Replica p receives and applies the next `count` factor sets of worker q, oldest first.
 * SFB_EINVAL (nothing applied) if p == q, or q has not produced that many, or it would break
 * the no-fast-forward rule. */
SFB_API sfb_status sfb_ssp_deliver(sfb_ssp *ssp, int32_t p, int32_t q, int32_t count);
/*
 * Partial broadcast (Section 4.3, Halton sequence broadcast): `sends` is a HOST P x P byte
 * matrix, sends[q*P + p] != 0 meaning worker q's factors go to replica p (the diagonal is
 * ignored).  The staleness rule then ranges over the workers that send to p, a delivery along
 * a missing edge is SFB_EINVAL, and the replicas no longer agree when everything has arrived.
 * Only before the first iteration (SFB_EINVAL afterwards).  Default: full broadcast.
 */
SFB_API sfb_status sfb_ssp_set_receivers(sfb_ssp *ssp, const uint8_t *sends);
/* The topology of Section 4.3: worker p sends to (p + floor(P h)) mod P for the first Q terms h
 * of 1/2, 1/4, 3/4, 1/8, 3/8, ... that give a new non-zero offset (at most P - 1 exist).
 * sends: HOST [P][P] bytes, overwritten.  SFB_EINVAL for P < 1, Q < 0 or a null pointer. */
SFB_API sfb_status sfb_halton_receivers(int32_t P, int32_t Q, uint8_t *sends);
/* Clocks: t [P] and tau [P][P] (row p = replica p), HOST int32 arrays; either may be NULL. */
SFB_API sfb_status sfb_ssp_state(const sfb_ssp *ssp, int32_t *t, int32_t *tau);

#ifdef __cplusplus
}
#endif
#endif /* SFB_H */
