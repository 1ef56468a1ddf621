/*
 * castling_attn.h -- C ABI of the MI355X (gfx950) linear-angular attention layer.
 *
 * The layer is the inference-time attention of Castling-ViT (arXiv 2211.10526,
 * Sec. 3.2.1).  Per (batch, head) unit with N tokens of width d it computes
 *
 *     q_hat_t = q_t / max(|q_t|, eps),  k_hat_j = k_j / max(|k_j|, eps)
 *     A_tj    = 1/2 + (q_hat_t . k_hat_j) / pi          linear terms of Eq. 8
 *     lin_t   = sum_j A_tj v_j / sum_j A_tj             Eq. 3 (row-sum normaliser)
 *     out_t   = lin_t + DWConv(V)_t                     Eq. 9 (sparse branch is 0 at inference)
 *
 * without ever forming A: it is reassociated (Sec. 3.1, kernel-based linear
 * attention) into the (d+1) x (d+1) state [K_hat | 1]^T [V | 1], i.e. K_hat^T V,
 * the K_hat column sum, the V column sum and N, followed by one q_hat . state
 * product per token.
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers unless a parameter says "host".
 *   - q, k, v, out: logical shape [B][heads][N][d], N = extra_tokens + grid_h * grid_w;
 *     the first extra_tokens tokens of a unit are not on the grid (class tokens), then
 *     grid token (y, x) is token extra_tokens + y * grid_w + x (row-major grid).  Tokens
 *     off the grid are keys and queries of the attention sums like any other; the DWConv
 *     term, defined on the grid, is zero for them and does not read them.  The d axis is always
 *     contiguous.  By default the tensors are contiguous in that order; the stride
 *     fields of the descriptor place them elsewhere, e.g. q, k, v as the three
 *     slices of a fused projection output [B][N][3][heads][d] (Sec. 3.1: Q, K, V are
 *     per-head linear projections of the same tokens) and out as [B][N][heads*d],
 *     the layout the output projection reads -- no permute copies on either side.
 *   - dw_weight: [heads][d][ks][ks] contiguous (one ks x ks filter per channel,
 *     shared over the batch); dw_bias: [heads][d] or NULL.
 *   - DWConv: zero "same" padding, stride 1, cross-correlation (no flip).
 *   - io_dtype is the type of q, k, v, dw_weight, dw_bias and out.  Accumulation
 *     is fp32 in all cases; bf16 and fp16 outputs are rounded to nearest even (fp16
 *     results beyond 65504 in magnitude become infinity).  bf16 and fp16 with d = 64, and
 *     with d = 32 where the head count is even, run on the matrix cores; fp32 and the
 *     other head widths run on the vector ALUs, at the next of the widths 16, 32, 64, 128
 *     with zero features in the gap (d = 96 costs about what d = 128 does).
 *   - The caller owns every tensor.  A handle owns only its workspace (partial
 *     states + final state), allocated by create and freed by destroy.
 *   - forward / reduce / apply only enqueue work on `stream` (a hipStream_t, NULL
 *     = the default stream) and never synchronise the host.  They may be called
 *     from several handles concurrently; one handle is not thread-safe.
 *   - Every function returns a castling_status_t (0 = OK).  Arguments are checked
 *     on the host before anything is launched; no exception crosses the boundary.
 *   - Results are run-to-run bitwise deterministic (no floating-point atomics).
 */
#ifndef CASTLING_ATTN_H
#define CASTLING_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct castling_attn* castling_attn_t; /* opaque, owned by the library */

typedef enum {
    CASTLING_OK = 0,
    CASTLING_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, N != extra_tokens + grid_h*grid_w, even ks, misalignment */
    CASTLING_ERR_UNSUPPORTED = 2, /* d, ks or dtype outside what the kernels are built for */
    CASTLING_ERR_HIP = 3,         /* a HIP runtime call failed (allocation, launch) */
    CASTLING_ERR_ALIAS = 4,       /* an output overlaps an input or another output */
    CASTLING_ERR_TOO_LARGE = 5    /* castling_attn_forward_static: more scratch memory needed than it holds */
} castling_status_t;

typedef enum { CASTLING_F32 = 0, CASTLING_BF16 = 1, CASTLING_F16 = 2 } castling_dtype_t;

typedef enum {
    CASTLING_NORM_ROWSUM = 0, /* divide by sum_j A_tj: the denominator of Eq. 3 (default) */
    CASTLING_NORM_NONE = 1    /* literal Eq. 9: Sim(Q,K) V with no denominator */
} castling_norm_t;

enum { CASTLING_BRANCH_LINEAR = 1, CASTLING_BRANCH_DWCONV = 2, CASTLING_BRANCH_ALL = 3 };

/* desc.flags.  KEEP_STATE: castling_attn_forward always leaves the fp32 state in the workspace
 * for castling_attn_get_state.  Without it a forward of a small problem does not spend memory
 * writes, or a launch, on a copy nobody reads.  castling_attn_reduce always leaves the state.
 * RESIDUAL_Q: the query as stored (not its unit row) is added to each output row after the
 * normaliser -- the residual connection of the pooled query in downsampling attention layers
 * (Sec. 3.1, attention designs; Table 1, last row).  Needs the linear branch
 * (CASTLING_ERR_INVALID_ARG otherwise); runs on the vector-ALU kernels.
 * TRAINING: create also allocates what castling_attn_backward needs (one more tensor of the
 * span of q, three of the span of k with q_pool = 2, and a few small buffers); shapes whose
 * backward tiles exceed the LDS of a block (fp32, d = 128, 9 x 9 filters) are refused with
 * CASTLING_ERR_UNSUPPORTED.
 * SEPARATE_PASSES: castling_attn_forward of a small problem (16-bit, d = 64, up to 256 tokens
 * per unit, filters up to 5 x 5) enqueues pass 1 and pass 2 as the separate launches castling_attn_reduce +
 * castling_attn_apply would, instead of its one-kernel form (for measurements and for tests
 * of those kernels; results agree to rounding).
 * VECTOR_ALU: 16-bit types stay on the vector-ALU kernels that fp32 uses (the fallback path;
 * for measurements and tests). */
enum {
    CASTLING_FLAG_KEEP_STATE = 1,
    CASTLING_FLAG_RESIDUAL_Q = 2,
    CASTLING_FLAG_TRAINING = 4,
    CASTLING_FLAG_SEPARATE_PASSES = 8,
    CASTLING_FLAG_VECTOR_ALU = 16
};

typedef struct {
    int32_t B, heads, N, d;   /* d: a multiple of 8, at most 128 */
    int32_t grid_h, grid_w;   /* N must equal extra_tokens + grid_h * grid_w */
    int32_t dw_kernel;        /* odd, 1..9 */
    int32_t io_dtype;         /* castling_dtype_t */
    int32_t norm;             /* castling_norm_t */
    uint32_t branches;        /* bitmask of CASTLING_BRANCH_*; 0 is read as CASTLING_BRANCH_ALL */
    float eps;                /* floor of the L2 norm; 0 is read as 1e-12; otherwise at least FLT_MIN */
    /* Element strides between consecutive batches, heads and tokens of q, k, v (one set for
     * all three) and of out.  All three of a set 0 = contiguous [B][heads][N][d], i.e.
     * {heads*N*d, N*d, d}.  Each must be a positive multiple of 16 bytes, the token stride at
     * least d.  N * token stride must stay below 4 GiB in bytes (with the default strides too: N * d
     * elements of a unit), else CASTLING_ERR_UNSUPPORTED.  The rows a set of strides
     * addresses must not overlap each other. */
    int64_t in_stride_b, in_stride_h, in_stride_n;
    int64_t out_stride_b, out_stride_h, out_stride_n;
    uint32_t flags;           /* bitmask of CASTLING_FLAG_* */
    int32_t extra_tokens;     /* tokens in front of the grid (class tokens), 0..64 */
    /* Downsampling layers (Sec. 3.1: queries pooled after their projection, K and V on every
     * token).  0 or 1: one query per token.  2: q and out hold Nq = ceil(grid_h/2) *
     * ceil(grid_w/2) tokens per unit, row-major over that coarser grid; query (y, x) stands at
     * position (2y, 2x) of the token grid, where its DWConv row is taken (a DWConv of stride 2;
     * the paper does not say how M_DW of Eq. 9 shrinks).  The pooling operator itself runs
     * before this library.  k, v keep N tokens and the in strides.  Runs on the vector-ALU
     * kernels in pass 2; extra_tokens must be 0 (CASTLING_ERR_UNSUPPORTED otherwise, as for
     * other values of q_pool, and for shapes whose tile of V exceeds the LDS of a block). */
    int32_t q_pool;
    int32_t reserved0;        /* must be 0 */
    /* q_pool = 2: element strides of q (rules as above; all 0 = contiguous [B][heads][Nq][d]);
     * the default of the out strides is then contiguous [B][heads][Nq][d] too.  Must be 0
     * otherwise (q shares the in strides). */
    int64_t q_stride_b, q_stride_h, q_stride_n;
} castling_attn_desc_t;

/* Host-only check of a descriptor (no GPU needed).  Sec. 3.2.1 fixes the shapes:
 * per head Q, K, V in R^{N x d}, DWConv over the token grid. */
int castling_attn_validate(const castling_attn_desc_t* desc);

/* Validates desc, allocates the workspace on the current device, returns a handle.  Every later
 * call on the handle must be made with that device current and with pointers into its memory;
 * calls on one handle must not overlap in time (its workspace holds the state between the two
 * passes), calls on different handles may. */
int castling_attn_create(const castling_attn_desc_t* desc, castling_attn_t* out_handle);

/* Whole layer (Eq. 9 with the readings above): reduce followed by apply.
 * q, k, v, dw_weight, out must be 16-byte aligned; out must not overlap q, k, v, the filters
 * or the bias (with strides the check compares the address ranges the tensors span, first to
 * last byte).  dw_weight may be NULL after castling_attn_prepare_weights: the filters
 * registered there are used. */
int castling_attn_forward(castling_attn_t h, const void* q, const void* k, const void* v,
                          const void* dw_weight, const void* dw_bias, void* out, void* stream);

/* castling_attn_forward for callers that cannot allocate device memory or keep a handle: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, checks and results as castling_attn_create(desc) + castling_attn_forward +
 * castling_attn_destroy (bitwise the same output: the same kernels run), but the workspace is
 * a fixed array of CASTLING_STATIC_SCRATCH_BYTES inside the library's device image, one copy
 * per GPU, held from the time the library is loaded on that GPU until the process ends.  The
 * call allocates and frees nothing on the device.
 *   - A problem whose workspace (castling_attn_workspace_bytes of a handle for desc) is larger
 *     is refused with CASTLING_ERR_TOO_LARGE before anything is enqueued; the five benchmark
 *     workloads fit.  CASTLING_FLAG_TRAINING is refused (CASTLING_ERR_INVALID_ARG); dw_weight
 *     must be given (there is no registration); the state cannot be fetched afterwards.
 *   - All calls on one GPU share that GPU's array, whatever their streams or threads: calls
 *     that overlap in time on one GPU race.  Nothing in the array needs clearing between
 *     calls: every call writes each part before it reads it, also after a call of another
 *     shape.
 *   - The first call on a device looks up the array's address, and a call with a descriptor
 *     other than the last one sets kernel attributes; make one call per descriptor outside
 *     graph capture first.  Repeated calls with the same descriptor only enqueue launches. */
#define CASTLING_STATIC_SCRATCH_BYTES (32u << 20)
int castling_attn_forward_static(const castling_attn_desc_t* desc, const void* q, const void* k,
                                 const void* v, const void* dw_weight, const void* dw_bias,
                                 void* out, void* stream);

/* First half: normalise K per token and reduce over tokens to the per-unit state
 * K_hat^T V, sum_j k_hat_j, sum_j v_j (Sec. 3.1 reassociation; sums of Eq. 3).
 * The state stays in the handle's workspace. */
int castling_attn_reduce(castling_attn_t h, const void* k, const void* v, void* stream);

/* Second half: normalise Q per token, apply the state the last castling_attn_reduce left in
 * the handle (Eq. 3 with the linear terms of Eq. 8), add DWConv(V) (Eq. 9), store out.
 * CASTLING_ERR_INVALID_ARG if the linear branch is on and the handle holds nothing to apply:
 * no reduce yet, or a castling_attn_forward since then that kept its state on chip.
 * dw_weight may be NULL after castling_attn_prepare_weights: the filters registered
 * there are used. */
int castling_attn_apply(castling_attn_t h, const void* q, const void* v, const void* dw_weight,
                        const void* dw_bias, void* out, void* stream);

/* Backward pass: the gradients of a scalar loss with respect to q, k, v, the DWConv filters and
 * their bias, given grad_out = dLoss/dout -- the derivatives of Eq. 9 (linear terms of Eq. 8,
 * normaliser of Eq. 3, DWConv term) with the readings above, for training the layer (Sec. 4.1;
 * the paper prints no gradient formulas).  The handle must have been created with
 * CASTLING_FLAG_TRAINING (CASTLING_ERR_INVALID_ARG otherwise).
 * grad_out has the type and strides of out; grad_q, grad_k, grad_v the type and strides of q, k,
 * v (with q_pool = 2, grad_out and grad_q hold one row per pooled query); grad_w [heads][d][ks][ks] and grad_bias [heads][d] (may be NULL) are fp32, contiguous, sums
 * over the batch.  All are overwritten, none accumulated into.  A branch that is off in the
 * descriptor contributes nothing: without the linear branch grad_q and grad_k are zeros,
 * without the DWConv branch grad_w and grad_bias (where given) are zeros and dw_weight may be
 * NULL.  With RESIDUAL_Q grad_q includes grad_out.  The forward pass is not needed
 * beforehand: pass 1 is recomputed.  Afterwards the handle holds no state to apply or fetch.
 * Pointers 16-byte aligned; no gradient (grad_w and grad_bias included) may overlap an input
 * or the filters, grad_w and grad_bias may not overlap any other gradient, and grad_q, grad_k,
 * grad_v must be three different pointers (CASTLING_ERR_ALIAS); their address ranges may
 * interleave, as slices of one fused [B][N][3][heads][d] gradient tensor do.  Only enqueues work on `stream`. */
int castling_attn_backward(castling_attn_t h, const void* q, const void* k, const void* v,
                           const void* dw_weight, const void* grad_out, void* grad_q, void* grad_k,
                           void* grad_v, float* grad_w, float* grad_bias, void* stream);

/* Registers the DWConv filters (the M_DW of Eq. 9) for later castling_attn_apply calls that
 * (and castling_attn_forward calls) that pass dw_weight = NULL, so that repeated calls with
 * fixed filters skip their per-call preparation.  The matrix-core path converts the filters into its operand table on
 * `stream` now (later changes to the buffer are not seen); the other paths keep the
 * pointer, which must stay valid and unchanged.  castling_attn_forward with dw_weight = NULL uses
 * the registration in the same way.  No other call on the handle (backward included) touches
 * the registered table; register again after the filters change. */
int castling_attn_prepare_weights(castling_attn_t h, const void* dw_weight, void* stream);

/* Training-time companions of the layer as O(N^2) attention on the matrix cores (16-bit I/O
 * with d = 64 and one query per token only, else CASTLING_ERR_UNSUPPORTED).  Shapes, strides and eps come from the handle.
 *   CASTLING_PAIR_SPARSE_SOFTMAX  out = Mask_thr(Softmax(scale * A B^T)) V, the auxiliary branch
 *       of Eq. 10 (Sec. 3.2.2).  Mask_thr(x) = x if x > thr else 0.  A, B = unit rows of q, k
 *       (normalize = 1, the rows the angular branch uses) or q, k themselves (normalize = 0);
 *       scale multiplies the logits (Eq. 10 prints none, Eq. 1 uses 1/sqrt(d)).
 *   CASTLING_PAIR_ANGULAR  out_t = sum_j A_tj v_j / sum_j A_tj with the exact angular kernel
 *       A_tj = 1 - arccos(q_hat_t . k_hat_j) / pi of Eq. 4-5 (the handle's norm: with
 *       CASTLING_NORM_NONE the division is left out); scale, threshold, normalize are ignored.
 * kept: DEVICE pointer to B*heads counters, or NULL; SPARSE_SOFTMAX writes the number of entries
 * the mask keeps per unit (the quantity whose decay to zero lets the branch be dropped at
 * inference).  out must not overlap q, k or v.
 * accumulate = 1 adds the result to what out already holds: castling_attn_forward followed by
 * SPARSE_SOFTMAX with accumulate = 1 on the same out gives the training-time attention with all
 * four terms of Eq. 9 (linear-angular terms, DWConv, and the masked softmax branch). */
typedef enum { CASTLING_PAIR_SPARSE_SOFTMAX = 0, CASTLING_PAIR_ANGULAR = 1 } castling_pair_mode_t;

typedef struct {
    int32_t mode;       /* castling_pair_mode_t */
    int32_t normalize;  /* SPARSE_SOFTMAX: 1 = unit rows, 0 = raw rows */
    float scale;        /* SPARSE_SOFTMAX: logit scale */
    float threshold;    /* SPARSE_SOFTMAX: mask threshold, in [0, 1] */
    int32_t accumulate; /* 0: out = result; 1: out += result (out is read, then rounded again) */
} castling_pair_params_t;

int castling_attn_pairwise(castling_attn_t h, const castling_pair_params_t* params, const void* q,
                           const void* k, const void* v, void* out, uint64_t* kept, void* stream);

/* NULL is a no-op returning CASTLING_OK. */
int castling_attn_destroy(castling_attn_t h);

/* Bytes of device workspace the handle holds. */
size_t castling_attn_workspace_bytes(castling_attn_t h);

/* Test/debug: copies the state of the last reduce to HOST memory as fp32
 * [B*heads][d+1][d+1] = [K_hat | 1]^T [V | 1] (row i < d: K_hat^T V row i then
 * ksum_i; row d: vsum then N).  Synchronises `stream`.  `bytes` must be exactly
 * B*heads*(d+1)*(d+1)*4.  CASTLING_ERR_INVALID_ARG if the workspace holds no state: nothing
 * has run yet, or the last call was a forward that never wrote the state to memory (small
 * problems keep it on chip, or sum its partial states inside the second pass) and the handle
 * was created without CASTLING_FLAG_KEEP_STATE. */
int castling_attn_get_state(castling_attn_t h, void* host_f32, size_t bytes, void* stream);

/* Number of token splits per unit the reduce uses for this handle (>= 1). */
int castling_attn_num_splits(castling_attn_t h);

/* Number of kernels one castling_attn_forward enqueues for this handle: 1 = the whole layer in
 * one kernel (state kept on chip), 2 = reduce + apply, 3 = reduce + combine + apply. */
int castling_attn_num_launches(castling_attn_t h);

/* Static string for a status code. */
const char* castling_attn_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* CASTLING_ATTN_H */
