/* mtpc.h - C ABI of libmtpc: the MtPC head (multi-token-prediction probabilistic
 * circuit head of a byte-level LLM) on one AMD MI355X (gfx950).
 *
 * For every position b the head maps a hidden vector h[b] (e_t in the paper) to
 * a joint distribution over the next n tokens, encoded by a probabilistic
 * circuit whose parameters are computed from h[b] (Sec. 3.3):
 *   input units   phi[b,i,j,:] = softmax(W[i,j] h[b])        W: [n][r][v][d]
 *   root weights  omega[b,:]   = softmax(Wsum h[b])          Wsum: [r][d]
 *   r x r sum layers (HMM transitions, binary-tree inner nodes): softmax over
 *   the last axis of caller-supplied logits (mtpc_sumlayers).
 * Circuit families (Sec. 2 and 3.2): fully factorised (Eq. FF, r must be 1),
 * CP mixture (Eq. CP), HMM (Eq. HMM), binary tree (Eq. BTree, n a power of two).
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller; the library
 *    allocates nothing, never synchronises and keeps nothing between calls that a
 *    result depends on (it remembers, per kernel and device, that the kernel's LDS
 *    limit has been raised; and the optional profiling events of a thread).
 *    Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *    default stream); buffers must stay alive until that work has completed.
 *  - Row-major, innermost axis contiguous.  h, W, Wsum share `dtype`
 *    (fp32, or bf16 with fp32 accumulation); all results are fp32 / int32.
 *  - h, W, Wsum and workspace must be 16-byte aligned; ld_h (row stride of h in
 *    elements) must keep rows 16-byte aligned and span at most 16 MiB; a row of W
 *    (d elements) at most 8 MiB.
 *  - Supported sizes: 1 <= B; d a multiple of 32; 1 <= n <= 64; 1 <= r <= 128;
 *    1 <= v <= 320.  Anything else returns MTPC_ERR_UNSUPPORTED.
 *  - Arguments are checked before the first launch: on MTPC_ERR_NULL, _SHAPE,
 *    _UNSUPPORTED and _WORKSPACE nothing has been enqueued and outputs are untouched.
 *    MTPC_ERR_HIP means the runtime refused a launch in the middle of a call: what
 *    was enqueued before it still runs, the outputs and the workspace are then
 *    unspecified.  Outputs are fully overwritten on success.
 *  - targets: int32, -1 marks a variable that is summed out (App. B.1: its input
 *    units integrate to 1); any other id outside [0, v) makes that row's outputs NaN.
 */
#ifndef MTPC_H
#define MTPC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MTPC_OK = 0,
  MTPC_ERR_NULL = 1,        /* a required pointer is NULL                     */
  MTPC_ERR_SHAPE = 2,       /* a size is non-positive or inconsistent         */
  MTPC_ERR_UNSUPPORTED = 3, /* outside the supported ranges listed above      */
  MTPC_ERR_WORKSPACE = 4,   /* workspace too small or misaligned              */
  MTPC_ERR_HIP = 5          /* a HIP launch reported an error                 */
} mtpc_status;

typedef enum { MTPC_F32 = 0, MTPC_BF16 = 1 } mtpc_dtype;
typedef enum { MTPC_FF = 0, MTPC_CP = 1, MTPC_HMM = 2, MTPC_BTREE = 3 } mtpc_family;
typedef enum { MTPC_OP_LOGLIK = 0, MTPC_OP_MARGINALS = 1, MTPC_OP_SAMPLE = 2, MTPC_OP_VERIFY = 3,
               MTPC_OP_BACKWARD = 4, MTPC_OP_TABLE = 5, MTPC_OP_WINDOWS = 6 } mtpc_op;
typedef enum { MTPC_MARG_PREFIX = 0, MTPC_MARG_UNIVARIATE = 1 } mtpc_marg_mode;
typedef enum { MTPC_SCORE_JOINT = 0, MTPC_SCORE_PREFIX = 1 } mtpc_score_mode;
typedef enum { MTPC_VERIFY_SAMPLING = 0, MTPC_VERIFY_GREEDY = 1 } mtpc_verify_mode;
typedef enum { MTPC_BWD_KEEP_PROBS = 0, MTPC_BWD_RECOMPUTE = 1 } mtpc_bwd_mode;

/* Common description of one call (Sec. 3.3). */
typedef struct {
  int32_t B, d, n, r, v;  /* positions, hidden size, window, units per layer, vocabulary */
  int32_t dtype;          /* mtpc_dtype of h, W, Wsum                                     */
  const void* h;          /* [B][ld_h] hidden states, first d entries of a row are used   */
  int64_t ld_h;           /* row stride of h in elements, >= d                            */
  const void* W;          /* [n][r][v][d] unembedding tensor                              */
  const void* Wsum;       /* [r][d] root mixture (CP, BTree) / initial state (HMM); NULL for FF */
  void* workspace;        /* device scratch, >= mtpc_workspace_bytes(...)                 */
  size_t workspace_bytes;
  void* stream;           /* hipStream_t                                                  */
  const void* W_stage_major; /* optional (NULL: none): the copy of W that mtpc_pack_weights makes.   */
                          /* The pass over all of W in mtpc_*_sample / *_greedy_draft /         */
                          /* *_loglik / *_marginals / *_window_scores / *_loss_backward reads it */
                          /* instead of W when its stages are the ones that pass uses: 128      */
                          /* bytes for B <= 64, 64 bytes for larger batches (same results, bit  */
                          /* for bit; 3-5 % less time), and so do the token draws of a larger   */
                          /* batch (each from its one slab; 64-byte stages, 6-8 % less time).   */
                          /* A copy with the other stage size is ignored.  W must be valid as   */
                          /* well: every other path reads W.                                    */
  int32_t W_stage_bytes;  /* stage size of that copy: 128 (also meant by 0) or 64               */
} mtpc_head;

/* r x r sum layers, normalised over the LAST axis (softmax), given either as
 * PRE-softmax fp32 logits or as the contextual parametrisation of Sec. 3.3.
 * HMM (Eq. HMM): L = n-1 transitions, logits[l][j][j'] scores z_{l+2}=j' given
 * z_{l+1}=j.  BTree (Eq. BTree): L = n-2, layer m-1 belongs to the inner node
 * with heap index m >= 1 (root 0, children 2m+1 / 2m+2, the leaf of token i at
 * n-1+i), logits[m-1][k][j] scores z_m=j given the parent's latent k.  A leaf's
 * r input units are indexed by its parent's latent; the root uses omega.
 * -inf logits are allowed (zero weight) as long as each row keeps one finite entry.
 *
 * Contextual layers (Sec. 3.3, sum unit parameters; App. HMM setup): when R is
 * non-NULL the logits of position b are  R[l][k][j][:] . h[b] + logits[l][k][j],
 * computed inside the library; `logits` is then the input-independent bias (NULL =
 * none; an identity bias - 0 on the diagonal, -inf off it - starts the circuit as
 * CP) and batch_stride must be 0.  R: [L][r][r][d] in the head's dtype, 16-byte
 * aligned, R_layer_stride = r*r*d, or 0 for one tensor shared by all layers. */
typedef struct {
  const float* logits;
  int64_t layer_stride;   /* r*r, or 0: one matrix shared by all L layers (homogeneous)   */
  int64_t batch_stride;   /* 0: shared by all positions; else elements between positions  */
  const void* R;          /* NULL: `logits` are the layer logits themselves               */
  int64_t R_layer_stride; /* elements between layers of R: r*r*d or 0                      */
} mtpc_sumlayers;

const char* mtpc_status_string(mtpc_status s);

/* Scratch needed by one call.  `layers` may be NULL (FF, CP).  `S` is the number
 * of drafts per position (sample) or of windows per position (MTPC_OP_TABLE,
 * MTPC_OP_WINDOWS: T + T2) and is ignored otherwise; `mode` is the
 * mtpc_marg_mode for MTPC_OP_MARGINALS and the mtpc_bwd_mode for MTPC_OP_BACKWARD.
 * Returns 0 for invalid arguments. */
size_t mtpc_workspace_bytes(int32_t family, int32_t op, const mtpc_head* head,
                            const mtpc_sumlayers* layers, int32_t S, int32_t mode);

/* Exact log-likelihood log q(x_1..x_n | context) of each position's target
 * window (Eqs. FF / CP / HMM / BTree; the circuit is normalised by
 * construction, App. B.1).  targets [B][n] int32 -> loglik [B] fp32. */
mtpc_status mtpc_ff_loglik(const mtpc_head* head, const int32_t* targets, float* loglik);
mtpc_status mtpc_cp_loglik(const mtpc_head* head, const int32_t* targets, float* loglik);
mtpc_status mtpc_hmm_loglik(const mtpc_head* head, const mtpc_sumlayers* T,
                            const int32_t* targets, float* loglik);
mtpc_status mtpc_btree_loglik(const mtpc_head* head, const mtpc_sumlayers* A,
                              const int32_t* targets, float* loglik);

/* Marginals (App. B.1: any subset of variables can be summed out exactly).
 * MTPC_MARG_PREFIX (Alg. 2, prefix marginals used by the accept test):
 *   out [B][n], out[b][i] = log q(x_1..x_{i+1}); out[b][n-1] is the log-likelihood.
 * MTPC_MARG_UNIVARIATE: out [B][n][v], out[b][i][a] = log q(x_{i+1} = a);
 *   targets is ignored and may be NULL.  The size mtpc_workspace_bytes returns has room for
 *   the input units of all positions (B n r v floats, when that is at most 8 GiB and r > 1):
 *   one pass writes them, a second kernel mixes them.  A workspace smaller by that many bytes
 *   is accepted too; the r units of a token are then mixed in registers (slower, above all
 *   for a few positions). */
mtpc_status mtpc_ff_marginals(const mtpc_head* head, const int32_t* targets, int32_t mode, float* out);
mtpc_status mtpc_cp_marginals(const mtpc_head* head, const int32_t* targets, int32_t mode, float* out);
mtpc_status mtpc_hmm_marginals(const mtpc_head* head, const mtpc_sumlayers* T,
                               const int32_t* targets, int32_t mode, float* out);
mtpc_status mtpc_btree_marginals(const mtpc_head* head, const mtpc_sumlayers* A,
                                 const int32_t* targets, int32_t mode, float* out);

/* Ancestral sampling (Alg. 1): S drafts per position.  Latents are drawn top
 * down from the sum-unit weights, then token i from the input unit selected by
 * the latent that indexes leaf i.  Every draw is an inverse-CDF search (smallest
 * k with u < p_0+..+p_k) on a uniform from Philox4x32-10 with key = (seed low,
 * seed high) and counter = (slot / 4, b, s, offset), output word slot % 4,
 * u = (word >> 8) * 2^-24.  Slots: token i -> i; latent l -> n + l with l = 0 for
 * the CP component, l = i for the HMM state z_{i+1}, l = m for the BTree node m.
 *   drafts      [B][S][n] int32 (required)
 *   latents     [B][S][n_lat] int32 or NULL; n_lat = 0 (FF), 1 (CP), n (HMM), n-1 (BTree)
 *   prefix_logq [B][S][n] fp32 or NULL: prefix marginals of each draft (as
 *               MTPC_MARG_PREFIX with the draft as target).
 *   logphi      [B][n][r][v] fp32 or NULL: the normalised input units
 *               log phi[b,i,j,:] = log softmax(W[i,j] h[b]) of every position, kept
 *               for the verification step (mtpc_*_verify) and mtpc_*_table_scores.
 * Batches of more than 64 positions evaluate only the input unit each token is drawn
 * from, unless logphi is requested or scores are wanted for fewer than 64 r drafts; so
 * do calls for a handful of drafts (2 B S <= r) that ask for neither scores nor logphi
 * (n B S rows of W are read instead of all n r v of them); a
 * draw whose uniform lies within rounding of a CDF step may then differ between calls
 * that ask for different outputs (the rule is the same, the fp32 partial sums are not). */
mtpc_status mtpc_ff_sample(const mtpc_head* head, int32_t S, uint64_t seed, uint32_t offset,
                           int32_t* drafts, int32_t* latents, float* prefix_logq, float* logphi);
mtpc_status mtpc_cp_sample(const mtpc_head* head, int32_t S, uint64_t seed, uint32_t offset,
                           int32_t* drafts, int32_t* latents, float* prefix_logq, float* logphi);
mtpc_status mtpc_hmm_sample(const mtpc_head* head, const mtpc_sumlayers* T, int32_t S,
                            uint64_t seed, uint32_t offset,
                            int32_t* drafts, int32_t* latents, float* prefix_logq, float* logphi);
mtpc_status mtpc_btree_sample(const mtpc_head* head, const mtpc_sumlayers* A, int32_t S,
                              uint64_t seed, uint32_t offset,
                              int32_t* drafts, int32_t* latents, float* prefix_logq, float* logphi);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): mtpc_*_sample with `family` as an argument (`layers` is
 * ignored for MTPC_FF / MTPC_CP and may be NULL) and with the scratch taken from a static
 * array of MTPC_STATIC_SCRATCH_BYTES in the library's device image instead of head->workspace
 * (head->workspace and workspace_bytes are ignored).  Nothing is allocated or freed by the call
 * or by anything it calls.  Every GPU the library runs on holds its own copy of the array from
 * load to process end; all calls on one GPU share it, so calls that overlap on one GPU - other
 * streams, other threads - race: issue them on one stream or order them yourself.  The array's
 * address on a device is looked up on the first call made with that device current (not a
 * stream operation; make that call outside a capture).
 * Sizes: whatever mtpc_*_sample accepts whose scratch fits: the sum-unit weights, the
 * normalised layers, latents, and - when prefix_logq is asked for - the evidence of the drafts,
 * about (B r + L r r + B S n (r + 3)) * 4 bytes.  A decode-sized batch (B <= 64) that asks for
 * prefix_logq must also pass logphi: the table of input units is then the caller's buffer, never
 * scratch.  Anything larger returns MTPC_ERR_WORKSPACE and launches nothing.
 * Results are those of mtpc_*_sample for the same arguments, bit for bit. */
#define MTPC_STATIC_SCRATCH_BYTES (4u << 20)
mtpc_status mtpc_sample_static(int32_t family, const mtpc_head* head, const mtpc_sumlayers* layers,
                               int32_t S, uint64_t seed, uint32_t offset, int32_t* drafts,
                               int32_t* latents, float* prefix_logq, float* logphi);

/* Scores of several windows per position in ONE unembedding pass: the log-likelihood
 * (Eqs. FF / CP / HMM / BTree) or the prefix marginals (Alg. 2) of every window, as
 * mtpc_*_loglik / MTPC_MARG_PREFIX compute them for one.  The windows come as two sets so
 * that, e.g., the targets and the drafts of the same positions are scored together
 * without copying them into one buffer:
 *   x  [B][T][n]  int32, T >= 1;   x2 [B][T2][n] int32 or NULL with T2 = 0;  -1 = summed out
 *   mode MTPC_SCORE_JOINT:  out [B][T+T2]     log q(window)
 *        MTPC_SCORE_PREFIX: out [B][T+T2][n]  prefix marginals
 *   (per position the T windows of x come first, then the T2 windows of x2)
 * Workspace: mtpc_workspace_bytes(family, MTPC_OP_WINDOWS, head, layers, T + T2, 0). */
mtpc_status mtpc_ff_window_scores(const mtpc_head* head, const int32_t* x, int32_t T,
                                  const int32_t* x2, int32_t T2, int32_t mode, float* out);
mtpc_status mtpc_cp_window_scores(const mtpc_head* head, const int32_t* x, int32_t T,
                                  const int32_t* x2, int32_t T2, int32_t mode, float* out);
mtpc_status mtpc_hmm_window_scores(const mtpc_head* head, const mtpc_sumlayers* T_layers,
                                   const int32_t* x, int32_t T, const int32_t* x2, int32_t T2,
                                   int32_t mode, float* out);
mtpc_status mtpc_btree_window_scores(const mtpc_head* head, const mtpc_sumlayers* A,
                                     const int32_t* x, int32_t T, const int32_t* x2, int32_t T2,
                                     int32_t mode, float* out);

/* Scores of arbitrary windows from the table of input units a sampling call left
 * (same head, same h): the evidence of each token is read from logphi and the circuit
 * is evaluated as in mtpc_*_loglik / MTPC_MARG_PREFIX (Eqs. FF / CP / HMM / BTree,
 * Alg. 2 prefix marginals), without another pass over W.  Serves the scoring of
 * several candidate windows per position, and - on a training-shaped batch - the
 * likelihood of the targets next to the drafts of the same positions from ONE
 * unembedding pass.
 *   logphi [B][n][r][v] fp32 (read only), as written by mtpc_*_sample / *_greedy_draft
 *   x      [B][T][n] int32 windows, -1 = summed out
 *   mode   MTPC_SCORE_JOINT: out [B][T] log q(x); MTPC_SCORE_PREFIX: out [B][T][n]
 * Workspace: mtpc_workspace_bytes(family, MTPC_OP_TABLE, head, layers, T, 0). */
mtpc_status mtpc_ff_table_scores(const mtpc_head* head, const float* logphi, const int32_t* x,
                                 int32_t T, int32_t mode, float* out);
mtpc_status mtpc_cp_table_scores(const mtpc_head* head, const float* logphi, const int32_t* x,
                                 int32_t T, int32_t mode, float* out);
mtpc_status mtpc_hmm_table_scores(const mtpc_head* head, const mtpc_sumlayers* T_layers,
                                  const float* logphi, const int32_t* x, int32_t T, int32_t mode,
                                  float* out);
mtpc_status mtpc_btree_table_scores(const mtpc_head* head, const mtpc_sumlayers* A,
                                    const float* logphi, const int32_t* x, int32_t T, int32_t mode,
                                    float* out);

/* Greedy draft for greedy speculative decoding (Sec. 3.4): the top-down traversal
 * of Alg. 1 with every draw replaced by the most likely outcome - each sum unit
 * takes its largest weight, each selected input unit its most likely token (ties:
 * the smallest index).  For the fully factorised head this is the exact mode of q;
 * for the other circuits it is a heuristic draft, which the greedy verification
 * corrects.  One draft per position: drafts [B][n]; latents, prefix_logq, logphi as
 * for mtpc_*_sample with S = 1 (any of them may be NULL).  Workspace: as for
 * MTPC_OP_SAMPLE with S = 1. */
mtpc_status mtpc_ff_greedy_draft(const mtpc_head* head, int32_t* drafts, int32_t* latents,
                                 float* prefix_logq, float* logphi);
mtpc_status mtpc_cp_greedy_draft(const mtpc_head* head, int32_t* drafts, int32_t* latents,
                                 float* prefix_logq, float* logphi);
mtpc_status mtpc_hmm_greedy_draft(const mtpc_head* head, const mtpc_sumlayers* T, int32_t* drafts,
                                  int32_t* latents, float* prefix_logq, float* logphi);
mtpc_status mtpc_btree_greedy_draft(const mtpc_head* head, const mtpc_sumlayers* A, int32_t* drafts,
                                    int32_t* latents, float* prefix_logq, float* logphi);

/* Verification step of one speculative-decoding cycle (Alg. 2 from the
 * acceptance loop on; greedy variant of Sec. 3.4), one draft per position.
 * Inputs (device): logphi [B][n][r][v] as written by mtpc_*_sample for the same
 * head; drafts [B][n] int32 in [0, v); prefix_logq [B][n] their prefix
 * marginals; p [B][n+1][v] fp32 verifier probabilities p(X_{t+i} | x_{<=t+i-1})
 * evaluated along the draft (rows sum to 1).
 * MTPC_VERIFY_SAMPLING: token s+1 is accepted unless alpha_s > p(x_{s+1}) /
 *   q(x_{s+1} | x_{<=s}), the conditional being exp(prefix_logq[s] -
 *   prefix_logq[s-1]); after the first rejection at position s one token is
 *   drawn from max(0, p[s] - q(. | x_{<=s})) / Z, where q(. | x_{<=s}) is the
 *   circuit's exact conditional over the whole vocabulary (if Z == 0, i.e.
 *   p == q, from p[s]); if all n are accepted the token is drawn from p[n].
 *   Uniforms: Philox as in mtpc_*_sample with slots 0..n-1 = alpha, slot n = the
 *   final draw, and the draft index s fixed at 2^32 - 1, which no drafting call
 *   uses: the same (seed, offset) as the call that drew the draft is safe.
 * MTPC_VERIFY_GREEDY: token s+1 is accepted iff it is argmax p[s] (ties: the
 *   smallest id); the emitted token is argmax p[accepted]; seed, offset, logphi
 *   and prefix_logq are unused and may be 0 / NULL.
 * Outputs: accepted [B] int32 in 0..n, token [B] int32: the token that follows
 * the accepted ones.  (A caller that shares the backbone state between draft and
 * verifier drops `token` whenever accepted > 0, App. speculative decoding.) */
mtpc_status mtpc_ff_verify(const mtpc_head* head, const float* logphi, const int32_t* drafts,
                           const float* prefix_logq, const float* p, int32_t mode, uint64_t seed,
                           uint32_t offset, int32_t* accepted, int32_t* token);
mtpc_status mtpc_cp_verify(const mtpc_head* head, const float* logphi, const int32_t* drafts,
                           const float* prefix_logq, const float* p, int32_t mode, uint64_t seed,
                           uint32_t offset, int32_t* accepted, int32_t* token);
mtpc_status mtpc_hmm_verify(const mtpc_head* head, const mtpc_sumlayers* T, const float* logphi,
                            const int32_t* drafts, const float* prefix_logq, const float* p,
                            int32_t mode, uint64_t seed, uint32_t offset, int32_t* accepted,
                            int32_t* token);
mtpc_status mtpc_btree_verify(const mtpc_head* head, const mtpc_sumlayers* A, const float* logphi,
                              const int32_t* drafts, const float* prefix_logq, const float* p,
                              int32_t mode, uint64_t seed, uint32_t offset, int32_t* accepted,
                              int32_t* token);

/* Training step (Sec. 4.1): the discounted, locally normalised negative
 * log-likelihood of overlapping windows and its gradients.  Token j (0-based) of
 * the window of position b contributes coef[b][j] * (-log q(x_j | x_<j)), the
 * conditional being a difference of prefix log-marginals:
 *   loss[b] = sum_j coef[b][j] * (P[b][j-1] - P[b][j]),   P[b][-1] = 0.
 * The caller folds gamma^j, the validity mask and the 1 / (N * V_ij) normalisation
 * of Eq. cross-ent-loss into coef [B][n] (fp32, device).  Outputs (device, fp32,
 * fully overwritten): loss [B]; gradients of sum_b loss[b]: dh [B][d] (row stride
 * d), dW [n][r][v][d], dWsum [r][d], dlayers = gradient w.r.t. the layer logits.
 * The logit gradient is kept in the dtype of h for the two contractions (bf16
 * inputs: rounded to nearest even).  Two plans, chosen by the workspace the call
 * is given: with mtpc_workspace_bytes(.., MTPC_OP_BACKWARD, .., mode =
 * MTPC_BWD_KEEP_PROBS) bytes the forward pass keeps its softmax probabilities
 * (n*r*v*B fp32) and the logit gradient is one elementwise pass; with the
 * smaller MTPC_BWD_RECOMPUTE size nothing of size n*r*v*B is kept in fp32 and the
 * logits are recomputed (one more pass of the unembedding product).
 * targets: ids in [0, v), or -1 (that variable is summed out and receives no
 * gradient).
 * dlayers has the shape of the stored layer logits ([n-1][r][r], or [1][r][r] for a
 * shared matrix, whose gradient is the sum over the steps).
 * Layers given per position (batch_stride != 0; dense [B][L or 1][r][r]): dlayers has
 * that shape too, the gradient w.r.t. each position's own logits.
 * Layers computed from h (mtpc_sumlayers.R non-NULL; R and bias either both one per
 * step / inner node, contiguous, or both shared by all of them): dR [L or 1][r][r][d]
 * receives the gradient w.r.t. R, dlayers the one w.r.t. the bias (may be NULL when
 * there is no bias), and dh includes the path through the layers; otherwise dR is
 * ignored and may be NULL.  Other stride combinations: MTPC_ERR_UNSUPPORTED.
 * Size limit of this call alone: a row of the logit gradient, n r v + r (+ L r r with R)
 * entries, and B, each at most 1,677,696 (beyond: MTPC_ERR_UNSUPPORTED). */
mtpc_status mtpc_ff_loss_backward(const mtpc_head* head, const int32_t* targets, const float* coef,
                                  float* loss, float* dh, float* dW);
mtpc_status mtpc_cp_loss_backward(const mtpc_head* head, const int32_t* targets, const float* coef,
                                  float* loss, float* dh, float* dW, float* dWsum);
mtpc_status mtpc_hmm_loss_backward(const mtpc_head* head, const mtpc_sumlayers* T, const int32_t* targets,
                                   const float* coef, float* loss, float* dh, float* dW, float* dWsum,
                                   float* dlayers, float* dR);
mtpc_status mtpc_btree_loss_backward(const mtpc_head* head, const mtpc_sumlayers* A,
                                     const int32_t* targets, const float* coef, float* loss, float* dh,
                                     float* dW, float* dWsum, float* dlayers, float* dR);

/* Stage-major copy of W for serving (W fixed between calls): per (i, j) slab, the S bytes
 * that each of the v rows contributes to a step along d lie back to back,
 *   W_stage_major [n*r][d * esz / S][v][S bytes]      (esz = 2 or 4 by head->dtype),
 * with S = head->W_stage_bytes (128, also meant by 0, or 64).  With 128-byte stages the pass that
 * streams W once (Sec. 3.3: all input units of a handful of positions, B <= 64, bound by the bytes
 * of W) reads long contiguous runs instead of 128 bytes from each of v rows d elements apart; with
 * 64-byte stages the pass of a larger batch asks the caches for whole lines instead of half lines.
 * Needs d * esz to be a multiple of S (else MTPC_ERR_UNSUPPORTED); uses head's d, n, r, v, dtype, W,
 * W_stage_bytes and stream only; W_stage_major is a device buffer of the size of W, 16-byte
 * aligned.  Hand it to later calls in mtpc_head.W_stage_major, with the same W_stage_bytes. */
mtpc_status mtpc_pack_weights(const mtpc_head* head, void* W_stage_major);

/* The uniforms the sampler consumes, out [B][S][slots] fp32 (device), for tests
 * of the generator and its slot map. */
mtpc_status mtpc_philox_uniforms(int32_t B, int32_t S, int32_t slots, uint64_t seed,
                                 uint32_t offset, float* out, void* stream);

/* Profiling aid (the only state the library keeps, per host thread): while both
 * events (hipEvent_t passed as void*) are non-NULL, every call made by this
 * thread records `start` right before and `stop` right after its unembedding
 * kernel launch(es) on the call's stream.  Pass NULLs to switch it off. */
void mtpc_profile_unembed(void* start_event, void* stop_event);
/* The same around the circuit kernel of a call (the sum / product layers of Eqs. FF / CP /
 * HMM / BTree on the evidence, with or without prefix marginals). */
void mtpc_profile_circuit(void* start_event, void* stop_event);

#ifdef __cplusplus
}
#endif
#endif /* MTPC_H */
