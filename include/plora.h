/*
 * plora.h - C ABI of the MI355X (gfx950) packed multi-LoRA linear layer, forward and backward.
 *
 * The layer (paper section 2.1 for LoRA, section 2.4 and appendix C.2 for packing): a frozen
 * weight W in R^{d_in x d_out} is shared by n_adapters LoRA adapters (A_k in R^{d_in x r_k},
 * B_k in R^{r_k x d_out}, multiplier scale_k = alpha_k / r_k chosen by the caller).  The tokens
 * of all adapters are stacked along the sequence dimension into x in R^{T x d_in}; segment s
 * holds rows seg_off[s] .. seg_off[s+1]-1 and belongs to adapter seg_adapter[s].  Row-vector
 * convention throughout:
 *
 *   forward   y_t  = x_t W + scale_k (x_t A_k) B_k                 t in a segment of adapter k
 *   backward  g_t  = scale_k dy_t B_k^T                            (appendix C.2, case 2)
 *             dx_t = dy_t W^T + g_t A_k^T                          (case 4)
 *             dA_k = sum_t x_t^T g_t                               (case 3)
 *             dB_k = scale_k sum_t (x_t A_k)^T dy_t                (case 1)
 *   W is frozen: no dW.
 *
 * General conventions
 *   - All matrices are dense row-major: x[T][d_in], W[d_in][d_out], A_k[d_in][r_k],
 *     B_k[r_k][d_out], y/dy[T][d_out], dx[T][d_in], dA_k[d_in][r_k], dB_k[r_k][d_out].
 *     With desc->w_layout = PLORA_W_OUT_IN the frozen weight alone is stored the other way round,
 *     W[d_out][d_in] (the layout of a framework's linear module: y = x W^T); everything else keeps
 *     the layouts above and every result is the same.
 *   - Pointers marked DEVICE point to memory of the current HIP device; pointers marked HOST are
 *     ordinary host memory that is read before the call returns (it may be freed afterwards).
 *   - The caller owns every buffer.  The library allocates no device memory; temporary storage
 *     comes from the caller's workspace (plora_workspace_bytes).
 *   - Calls only enqueue work on the given HIP stream (a hipStream_t passed as void*; NULL is
 *     the default stream) and never synchronise.  Two calls that share a workspace must be
 *     ordered on one stream.
 *   - Every argument is validated before anything is enqueued; on error nothing is launched and
 *     no output is touched.  No exception or abort crosses this boundary (a failed host
 *     allocation comes back as PLORA_ERR_INTERNAL).
 *   - Thread safety: calls may come from several host threads and on several devices (the current
 *     HIP device of the calling thread is used); the only state the library keeps is a small
 *     cache of derived metadata keyed by the description and per-device launch set-up, both behind
 *     locks.  Calls that share a workspace must be ordered on one stream.
 *   - x, W, A_k, B_k, y, dy, dx have the element type desc->dtype.  The saved low-rank
 *     activation h and the gradients dA_k, dB_k are always fp32.  bf16 results are rounded to
 *     nearest-even from fp32 accumulators.
 */
#ifndef PLORA_H
#define PLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PLORA_MAX_RANK      128   /* the paper's rank range ends at 128 (Table 1)              */
#define PLORA_MAX_ADAPTERS  256
#define PLORA_MAX_SEGMENTS 1024
#define PLORA_MAX_GROUP       4   /* projections per grouped call (q / k / v; gate / up)          */

typedef enum {
    PLORA_OK = 0,
    PLORA_ERR_NULL = 1,         /* a required pointer is NULL                                   */
    PLORA_ERR_SHAPE = 2,        /* T, d_in or d_out negative / zero / not a multiple of 8 (bf16),
                                   d_in or d_out above 2^22, T above 2^31 - 1, more than 2^30
                                   256 x 256 output tiles, fp32 with T above 65535 * 64          */
    PLORA_ERR_SEGMENTS = 3,     /* offsets do not start at 0, end at T, or decrease             */
    PLORA_ERR_ADAPTER = 4,      /* adapter id outside [-1, n_adapters) or too many of them      */
    PLORA_ERR_RANK = 5,         /* rank outside [1, PLORA_MAX_RANK]                             */
    PLORA_ERR_ALIGN = 6,        /* a device pointer is not 16-byte aligned                      */
    PLORA_ERR_WORKSPACE = 7,    /* workspace NULL or smaller than plora_workspace_bytes()       */
    PLORA_ERR_UNSUPPORTED = 8,  /* unknown dtype or weight layout                               */
    PLORA_ERR_HIP = 9,          /* a HIP call failed (launch error)                             */
    PLORA_ERR_INTERNAL = 10,    /* host memory allocation failed or another internal error      */
    PLORA_ERR_GROUP = 11        /* grouped call: n_proj outside [1, PLORA_MAX_GROUP], the projections
                                   differ in dtype, T, d_in, segments or adapters, or both dx and
                                   dx_sum are given                                              */
} plora_status;

typedef enum { PLORA_BF16 = 0, PLORA_F32 = 1 } plora_dtype;

/* Storage of the frozen weight. */
typedef enum {
    PLORA_W_IN_OUT = 0,         /* W[d_in][d_out]: rows are input features                         */
    PLORA_W_OUT_IN = 1          /* W[d_out][d_in]: rows are output features (y = x W^T)            */
} plora_w_layout;

/* Shape and packing of one call.  Every array here is HOST memory. */
typedef struct {
    int64_t T;                    /* total tokens (rows of x); 0 is legal                       */
    int64_t d_in;                 /* d of the paper                                             */
    int64_t d_out;                /* k of the paper                                             */
    int32_t n_seg;                /* number of segments, 0 only if T == 0                       */
    int32_t n_adapters;
    const int32_t *seg_off;       /* [n_seg+1] nondecreasing, seg_off[0]=0, seg_off[n_seg]=T    */
    const int32_t *seg_adapter;   /* [n_seg] in [0, n_adapters), or -1: base weight only        */
    const int32_t *rank;          /* [n_adapters] r_k in [1, PLORA_MAX_RANK]                    */
    const float *scale;           /* [n_adapters] scale_k                                       */
    int32_t dtype;                /* plora_dtype of x, W, A, B, y, dy, dx                       */
    int32_t w_layout;             /* plora_w_layout of W                                        */
} plora_desc;

/* Text for a status code (static storage, never NULL). */
const char *plora_status_string(plora_status st);

/* Validates a description (host only, touches no device).  Returns PLORA_OK or the error. */
plora_status plora_validate(const plora_desc *desc);

/*
 * Number of fp32 elements of the saved low-rank activation: sum over segments of
 * (segment length x rank of its adapter); segments of adapter -1 contribute nothing.
 * Segment s starts at the prefix sum of the segments before it and is stored [length][r_k]
 * row-major.  Returns 0 for an invalid description.
 */
size_t plora_h_elems(const plora_desc *desc);

/* Bytes of DEVICE workspace that plora_linear_fwd and plora_linear_bwd need for this
 * description (the larger of the two; 256-byte aligned base expected).  0 if invalid. */
size_t plora_workspace_bytes(const plora_desc *desc);

/*
 * Layout of the saved activation and a token-block view of the packing (host only; what a caller
 * needs to address h_saved, and a simple form of the segment table for tests).  The tables the
 * kernels themselves read are exported by plora_debug_metadata (plora_debug.h).
 *   h_off_out   [n_seg+1] element offset of each segment inside the saved activation
 *               (int64 prefix sums of length x rank); may be NULL.
 *   blocks_out  token blocks of at most block_rows rows that never straddle a segment, in row
 *               order, 4 int32 each: {first row, number of rows, segment, adapter}; empty
 *               segments produce none.  Written up to blocks_cap entries; may be NULL.
 * Returns the number of token blocks (also when blocks_out is NULL or too small), or -1 for an
 * invalid description or block_rows < 1.
 */
int64_t plora_build_metadata(const plora_desc *desc, int32_t block_rows, int64_t *h_off_out,
                             int32_t *blocks_out, int64_t blocks_cap);

/*
 * Forward (section 2.4; y_t = x_t W + scale_k (x_t A_k) B_k).
 *   x        DEVICE [T][d_in]
 *   W        DEVICE [d_in][d_out], or [d_out][d_in] with PLORA_W_OUT_IN
 *   A, B     HOST arrays of n_adapters DEVICE pointers, A[k] -> [d_in][r_k], B[k] -> [r_k][d_out]
 *   y        DEVICE [T][d_out], overwritten
 *   h_saved  DEVICE fp32 [plora_h_elems] or NULL; if given it receives x_t A_k for every
 *            token (layout above) for later use by plora_linear_bwd
 *   workspace, ws_bytes  DEVICE scratch, at least plora_workspace_bytes(desc)
 */
plora_status plora_linear_fwd(const plora_desc *desc, const void *x, const void *W,
                              const void *const *A, const void *const *B, void *y,
                              float *h_saved, void *workspace, size_t ws_bytes, void *hip_stream);

/*
 * Forward for callers that cannot allocate device memory and have no workspace to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error codes as plora_linear_fwd, without the workspace: the temporary
 * storage is a scratch array of PLORA_NOALLOC_SCRATCH_BYTES that is part of the library's device
 * image (one copy per GPU, held until the process ends).  The call allocates and frees nothing.
 * A description whose plora_workspace_bytes exceeds the scratch size is refused with
 * PLORA_ERR_WORKSPACE before anything is enqueued.  Every call on one GPU uses that GPU's one
 * array (it keeps the previous call's contents; the call rewrites what it reads), so calls of
 * this entry point that overlap on one GPU - different streams, or different host threads - race;
 * order them on one stream.
 */
#define PLORA_NOALLOC_SCRATCH_BYTES (64u << 20)
plora_status plora_linear_fwd_noalloc(const plora_desc *desc, const void *x, const void *W,
                                      const void *const *A, const void *const *B, void *y,
                                      float *h_saved, void *hip_stream);

/*
 * Backward (appendix C.2, cases 1-4; no gradient for W).
 *   x, W, A, B as in the forward call;  dy DEVICE [T][d_out]
 *   h_saved  DEVICE fp32 activation written by the forward call with the same inputs, or NULL
 *            (then x_t A_k is recomputed)
 *   dx       DEVICE [T][d_in], overwritten; NULL skips it
 *   dA, dB   HOST arrays of n_adapters DEVICE fp32 pointers, dA[k] -> [d_in][r_k],
 *            dB[k] -> [r_k][d_out]; overwritten (an adapter without tokens gets zeros; several
 *            segments of one adapter are summed).  Both NULL skips the weight gradients.
 */
plora_status plora_linear_bwd(const plora_desc *desc, const void *x, const void *W,
                              const void *const *A, const void *const *B, const void *dy,
                              const float *h_saved, void *dx, float *const *dA,
                              float *const *dB, void *workspace, size_t ws_bytes,
                              void *hip_stream);

/*
 * Stand-alone low-rank update, for callers that compute the base product themselves (another GEMM library, a
 * quantised weight): the packed LoRA kernels beside the framework's base GEMM, as the paper runs them (section 2.4,
 * appendix C.2).  Same packing, arguments and error codes as the fused calls, without W (desc->w_layout is not used):
 *   plora_lora_fwd   y_t  += scale_k (x_t A_k) B_k     y  DEVICE [T][d_out], holds x W on entry, updated in place
 *   plora_lora_bwd   dx_t += g_t A_k^T                 dx DEVICE [T][d_in], holds dy W^T on entry; NULL skips it
 *                    dA_k, dB_k as plora_linear_bwd (overwritten)
 * Rows of segments without an adapter are left as they are.  The sum is formed in fp32 (fp64 for PLORA_F32) and
 * rounded once.  The workspace must hold plora_lora_workspace_bytes(desc) bytes (0 for an invalid description).
 */
size_t plora_lora_workspace_bytes(const plora_desc *desc);
plora_status plora_lora_fwd(const plora_desc *desc, const void *x, const void *const *A, const void *const *B,
                            void *y, float *h_saved, void *workspace, size_t ws_bytes, void *hip_stream);
plora_status plora_lora_bwd(const plora_desc *desc, const void *x, const void *const *A, const void *const *B,
                            const void *dy, const float *h_saved, void *dx, float *const *dA, float *const *dB,
                            void *workspace, size_t ws_bytes, void *hip_stream);

/*
 * Several projections on one x (q / k / v of an attention block, gate / up of an MLP): appendix C.2's concatenation of
 * the adapters into one tensor, applied across the projections that share an input.  Projection p is an ordinary
 * layer of its own - its W_p, d_out, ranks r_{k,p}, scales, A_{k,p}, B_{k,p}, weight layout - and every result is what
 * plora_linear_fwd / _bwd give for it alone.  What is shared is the traffic: x_t A_{k,p} for all p comes from one pass
 * over x against the A_{k,p} laid side by side, and dA_{k,p} for all p from one pass over x against the g_{t,p} laid
 * side by side.  Projections are fused as long as their ranks, each rounded up to a multiple of 16, sum to at most
 * PLORA_MAX_RANK for every adapter; a group beyond that is cut into several fused passes, in the order given.
 *   group->desc   HOST array of n_proj descriptions with the same dtype, T, d_in, n_seg, seg_off, seg_adapter and
 *                 n_adapters (PLORA_ERR_GROUP otherwise)
 *   W, y, dy, dx, h_saved   HOST arrays of n_proj DEVICE pointers, entry p as in the plain call for projection p
 *                 (dx, h_saved: the array or single entries may be NULL; dx[p] is projection p's own dy_p W_p^T +
 *                 g_p A_p^T)
 *   dx_sum        DEVICE [T][d_in] or NULL: the gradient of the shared input, sum over p of dy_p W_p^T + g_p A_p^T
 *                 (case 4 of appendix C.2 for every projection that reads x).  Projection 0 overwrites it, every
 *                 further projection's GEMM adds to it in its epilogue, so no projection's own dx is ever stored;
 *                 in bf16 the running sum is rounded after every projection, as a chain of bf16 additions would.
 *                 Give dx or dx_sum, not both (PLORA_ERR_GROUP)
 *   A, B, dA, dB  HOST arrays of n_proj HOST arrays of n_adapters DEVICE pointers; dA / dB: the array, or entry p of
 *                 both, may be NULL (no weight gradients for that projection)
 * The workspace must hold plora_group_workspace_bytes(group) bytes (0 for an invalid group).  PLORA_F32 groups are
 * accepted and run projection by projection.
 */
typedef struct {
    int32_t n_proj;               /* 1 .. PLORA_MAX_GROUP                                          */
    const plora_desc *desc;       /* HOST [n_proj]                                                  */
} plora_group;
size_t plora_group_workspace_bytes(const plora_group *group);
plora_status plora_group_fwd(const plora_group *group, const void *x, const void *const *W,
                             const void *const *const *A, const void *const *const *B, void *const *y,
                             float *const *h_saved, void *workspace, size_t ws_bytes, void *hip_stream);
plora_status plora_group_bwd(const plora_group *group, const void *x, const void *const *W,
                             const void *const *const *A, const void *const *const *B, const void *const *dy,
                             const float *const *h_saved, void *const *dx, void *dx_sum,
                             float *const *const *dA, float *const *const *dB, void *workspace, size_t ws_bytes,
                             void *hip_stream);

/*
 * The layer on a base weight stored as 4-bit NormalFloat (NF4, the storage QLoRA publishes; the paper applies packed
 * LoRA to such a base and notes that the LoRA computation does not change).  Storage of W, flat in the memory order
 * that desc->w_layout names: blocks of 64 consecutive elements; per block one fp32 constant (its largest magnitude);
 * per element a 4-bit index into the 16 levels of the format, two per byte, the element with the even position in the
 * high half.  An element is level[index] * constant, formed in fp32 and, for PLORA_BF16, rounded to nearest even.
 *   W_codes   DEVICE [d_in * d_out / 2] bytes, 16-byte aligned
 *   W_absmax  DEVICE [d_in * d_out / 64] fp32, 16-byte aligned
 * d_in * d_out must be a multiple of 64 (PLORA_ERR_SHAPE otherwise).
 *
 * plora_nf4_dequantize writes the n_elems values (a multiple of 64; dtype: plora_dtype of `out`) and is all a caller
 * needs who wants to keep the expanded weight.  plora_linear_fwd_nf4 / _bwd_nf4 are plora_linear_fwd / _bwd on the
 * stored weight: they expand W into the workspace first (the backward call only if dx is wanted), so the workspace
 * must hold plora_nf4_workspace_bytes(desc) bytes; everything else is as for those calls.
 */
size_t plora_nf4_workspace_bytes(const plora_desc *desc);
plora_status plora_nf4_dequantize(const void *W_codes, const float *W_absmax, int64_t n_elems, int32_t dtype,
                                  void *out, void *hip_stream);
plora_status plora_linear_fwd_nf4(const plora_desc *desc, const void *x, const void *W_codes, const float *W_absmax,
                                  const void *const *A, const void *const *B, void *y, float *h_saved,
                                  void *workspace, size_t ws_bytes, void *hip_stream);
plora_status plora_linear_bwd_nf4(const plora_desc *desc, const void *x, const void *W_codes, const float *W_absmax,
                                  const void *const *A, const void *const *B, const void *dy, const float *h_saved,
                                  void *dx, float *const *dA, float *const *dB, void *workspace, size_t ws_bytes,
                                  void *hip_stream);

/*
 * Per-adapter optimizer step after a backward call (section 2.4: every adapter keeps its own
 * parameters and optimizer state; appendix B: AdamW with gradient, momentum and velocity per
 * adapter; Table 1: the learning rate is a per-job hyperparameter).  AdamW as published, in the
 * order the common frameworks apply it, for every element of A_k and B_k of every adapter k:
 *     g <- grad_scale_k g
 *     theta <- theta (1 - lr_k wd_k);  m <- beta1_k m + (1 - beta1_k) g;  v <- beta2_k v + (1 - beta2_k) g^2
 *     theta <- theta - lr_k (m / (1 - beta1_k^t_k)) / (sqrt(v / (1 - beta2_k^t_k)) + eps_k)
 * fp32 arithmetic.  The parameter proper is the fp32 master copy; the copy in the layer's I/O type
 * (what plora_linear_fwd / _bwd read) is rewritten from it, bf16 rounded to nearest even.
 */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int32_t step;                 /* t of this update: 1 for the adapter's first step                */
    float grad_scale;             /* multiplier on the adapter's gradient before the rule, g <- grad_scale g:
                                     every adapter has its own data and loss (section 2.4), so the factor
                                     that normalises by its own batch size (a per-job knob, Table 1) or
                                     clips by its own gradient norm is per adapter.  1 for none; finite   */
} plora_adamw_hparams;

/* One side (all A_k, or all B_k): HOST arrays of n_adapters DEVICE pointers, 16-byte aligned,
 * each tensor in the shape of A_k ([d_in][r_k]) or B_k ([r_k][d_out]). */
typedef struct {
    void *const *param;           /* desc->dtype copy, overwritten.  NULL table: no copy is kept     */
    float *const *master;         /* fp32 parameters, updated in place.  NULL table: only for
                                     PLORA_F32, then param itself is the parameter                   */
    const float *const *grad;     /* fp32 gradients as written by plora_linear_bwd                   */
    float *const *m;              /* fp32 first moment, updated in place                             */
    float *const *v;              /* fp32 second moment, updated in place                            */
} plora_adamw_side;

/*
 * Enqueues the update of every adapter on the stream (one or two launches per 40 tensors; no
 * workspace).  Only T-independent parts of desc are used: d_in, d_out, n_adapters, rank, dtype
 * (the description is validated as a whole).  hp: HOST array of n_adapters.  Errors as for the
 * other calls: PLORA_ERR_NULL for a missing table or pointer (param and master both absent, master
 * absent with bf16), PLORA_ERR_ALIGN, PLORA_ERR_SHAPE for step < 1, betas outside [0, 1) or a
 * grad_scale that is not finite.
 */
plora_status plora_adamw_step(const plora_desc *desc, const plora_adamw_side *A, const plora_adamw_side *B,
                              const plora_adamw_hparams *hp, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PLORA_H */
