/*
 * blstm_mi355 -- one learner's training step for a bidirectional-LSTM acoustic
 * model, and the ADPSGD pairwise weight-averaging step, as HIP kernels for gfx950.
 *
 * The calls follow the paper's own statement of the problem:
 *   g  = calGrad(W)    (section 3.2)  = blstm_forward + softmax_xent_fwd_bwd + blstm_backward
 *   W' = apply(W, g)   (section 3.2, Eq. 1c) = sgd_step
 *   theta_i <- (theta_i' + theta_j')/2 (Eq. 4, second line) = adpsgd_mix
 *
 * Model (section 4.2): L bidirectional LSTM layers with H cells per direction, the
 * two directions concatenated; a linear bottleneck of P units; a softmax over V
 * classes; sequences unrolled over T frames with zero initial state.
 *
 * Conventions common to every call
 *   - Every pointer named theta, x, z, dz, grad, labels, loss, velocity or workspace is
 *     DEVICE memory owned by the caller.  The library never allocates or frees
 *     device memory and never synchronises the device: all work is enqueued on the
 *     caller's stream (a hipStream_t passed as void*, NULL = the null stream).
 *   - `partner` and every `*_out` size/offset argument is HOST memory.
 *   - Activations are time-major and row-major: [T][B][features].
 *   - mode 0: every tensor is float.  mode 1: theta, x, z, dz are bfloat16 (the
 *     bf16 shadow of the weights; RNE rounding), products accumulate in float,
 *     gradients, the loss, the master weights and the velocity are float.
 *   - Return value: 0 on success, otherwise one of the negative codes below; the
 *     text is available from blstm_last_error().  Arguments are validated before
 *     the first launch, so a call that fails validation has no side effects.
 *   - Flat parameter layout (elements, row-major, gate blocks in the order i,f,g,o):
 *       for layer l = 0..L-1, for direction d in (0 = forward, 1 = backward):
 *           W_x [4H][D_l], U_h [4H][H], b [4H]      D_0 = D, D_l = 2H for l > 0
 *       W_p [P][2H], b_p [P]                        absent when P == 0
 *       W_s [V][P or 2H], b_s [V]
 *     blstm_param_offset reports where each tensor sits.
 */
#ifndef BLSTM_MI355_H
#define BLSTM_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BLSTM_OK              0
#define BLSTM_ERR_NULL       -1   /* a required pointer is NULL */
#define BLSTM_ERR_DIM        -2   /* bad dimension or unsupported configuration */
#define BLSTM_ERR_WORKSPACE  -3   /* workspace not bound or too small */
#define BLSTM_ERR_ALIGN      -4   /* pointer not aligned to 16 bytes */
#define BLSTM_ERR_HIP        -5   /* a HIP call failed */

/* which = one of these in blstm_param_offset */
#define BLSTM_WX 0
#define BLSTM_UH 1
#define BLSTM_B  2
#define BLSTM_WP 3
#define BLSTM_BP 4
#define BLSTM_WS 5
#define BLSTM_BS 6

#define BLSTM_MAX_REPLICAS 64

typedef struct blstm_ctx blstm_ctx;            /* opaque, host only; owns no device memory */

typedef struct {
    int32_t T, B, D, H, L, P, V;               /* P == 0: no bottleneck, the softmax reads the LSTM output */
    int32_t mode;                              /* 0 = fp32, 1 = bf16 storage + fp32 accumulation */
    float   loss_scale;                        /* s of E = s * sum_frames -log p[label]; <= 0: 1/(T*B) (Eq. 1a) */
} blstm_config;

/* Context: shapes, parameter layout, workspace layout.  Host-side only. */
int    blstm_create(const blstm_config* cfg, blstm_ctx** out);
void   blstm_destroy(blstm_ctx* ctx);
size_t blstm_param_count(const blstm_ctx* ctx);           /* N: elements of theta and of grad; 0 if ctx is NULL */
size_t blstm_workspace_bytes(const blstm_ctx* ctx);       /* saved activations + scratch for one step */
/* Offset and length (elements) of one tensor in the flat vector.  layer/dir are ignored for which >= BLSTM_WP. */
int    blstm_param_offset(const blstm_ctx* ctx, int layer, int dir, int which, size_t* off_out, size_t* len_out);
/* Hands the library `bytes` of caller-owned device memory (16-byte aligned) to keep between
   blstm_forward and blstm_backward.  The contents need no initialisation. */
int    blstm_bind(blstm_ctx* ctx, void* workspace, size_t bytes);

/* Forward pass of the LSTM stack and the bottleneck (section 4.2).
   theta [N], x [T][B][D] -> z_out [T][B][P or 2H]; activations for BPTT are kept in the workspace. */
int blstm_forward(blstm_ctx* ctx, const void* theta, const void* x, void* z_out, void* stream);

/* Softmax cross-entropy over V classes (Eq. 1a with the frame-level criterion) and its gradients:
   loss_dev[0] = s * sum -log p[label]; dz = dE/dz [T][B][P or 2H];
   grad: only the W_s and b_s slices are written (overwritten, not accumulated).
   labels [T][B] int32 in [0, V).  A label outside that range is never used as an index: its frame's loss term, and
   with it the loss, becomes NaN. */
int softmax_xent_fwd_bwd(blstm_ctx* ctx, const void* theta, const void* z, const int32_t* labels,
                         float* loss_dev, void* dz, float* grad, void* stream);

/* softmax_xent_fwd_bwd for callers that cannot allocate device memory or bind a workspace at that point
   (code under stream capture, tight serving loops, harnesses that forbid allocation): same arguments, same
   kernels and same results, but the scratch of the call (the logit matrix [T*B][V] in the storage type, one
   loss term per frame, partial tiles of the products split along the contraction) lives in an array of
   BLSTM_NOALLOC_SCRATCH_BYTES inside the library's code object instead of the bound workspace; no workspace
   needs to be bound.  Each GPU the library runs on holds that array until the process ends.  The call
   allocates and frees nothing.  Shapes whose scratch exceeds the array are rejected with
   BLSTM_ERR_WORKSPACE before any launch (roughly T*B*V*2 bytes in mode 1, *4 in mode 0, plus a few MB).
   All calls on one GPU share the array: calls that overlap on one GPU (different streams or threads) race;
   everything the call reads from the array it has written itself earlier in the same call. */
#define BLSTM_NOALLOC_SCRATCH_BYTES (32u << 20)
int softmax_xent_fwd_bwd_noalloc(blstm_ctx* ctx, const void* theta, const void* z, const int32_t* labels,
                                 float* loss_dev, void* dz, float* grad, void* stream);

/* Back-propagation through the bottleneck and through time (Eq. 1b): writes every slice of grad
   except W_s and b_s.  Must follow blstm_forward on the same ctx, theta and x. */
int blstm_backward(blstm_ctx* ctx, const void* theta, const void* x, const void* dz, float* grad, void* stream);

/* Eq. 1c: theta <- theta - lr * grad over n elements.  With momentum != 0 (velocity required):
   v <- momentum * v + grad; theta <- theta - lr * v.  theta_bf16, if not NULL, receives the
   RNE-rounded bf16 copy of the updated weights in the same pass. */
int sgd_step(float* theta_master, void* theta_bf16_or_null, const float* grad, size_t n,
             float lr, float momentum, float* velocity_or_null, void* stream);

/* Eq. 4, second line, for one matching of R replicas: for every pair {i, partner[i]} both members
   become (theta_i + theta_j)/2; partner[i] == i leaves replica i untouched.
   theta_master: HOST array of R device pointers (n floats each); theta_bf16_or_null: HOST array of R
   device pointers to the bf16 copies, or NULL; partner: HOST array, must be an involution. R <= 64. */
int adpsgd_mix(float* const* theta_master, void* const* theta_bf16_or_null, size_t n, int R,
               const int32_t* partner, void* stream);

/* Eq. 1c and Eq. 4 (second line) for one pair in a single pass: theta_i' = theta_i - lr grad_i and
   theta_j' = theta_j - lr grad_j (momentum as in sgd_step, each replica with its own velocity), then both
   replicas become (theta_i' + theta_j')/2.  Same arithmetic, element by element, as sgd_step on each
   replica followed by adpsgd_mix on the pair; the weights are read and written once instead of twice.
   All pointers are device pointers, 16-byte aligned, n elements; the bf16 copies are both given or both NULL.
   grad_j == NULL: replica j takes no update in this call (the learner that owns it has applied its own, Eq. 4's
   first factor) and enters the average as it stands; velocity_j is then ignored.  This is one learner's
   sgd_step followed by its adpsgd_mix with a neighbour, in one pass. */
int sgd_mix_pair(float* theta_i, float* theta_j, void* theta_bf16_i_or_null, void* theta_bf16_j_or_null,
                 const float* grad_i, const float* grad_j, size_t n, float lr, float momentum,
                 float* velocity_i_or_null, float* velocity_j_or_null, void* stream);

/* The synchronous strategy of section 3.2 (Fig. 3a: W = allreduce(W') / lambda) for R replicas held in one
   GPU's memory: every replica becomes the mean of all R, summed in the order 0..R-1 in float and scaled
   by 1/R.  theta_master / theta_bf16_or_null: HOST arrays of R device pointers as for adpsgd_mix. */
int sync_average(float* const* theta_master, void* const* theta_bf16_or_null, size_t n, int R, void* stream);

/* Learning rate of a 1-based epoch under section 3.1's recipe (host arithmetic, no device work): linear
   warm-up from base_lr to peak_lr over the first warmup_epochs epochs, then a factor 1/sqrt(2) per epoch
   from epoch anneal_from on.  The paper's runs: warmup_epochs = 10, anneal_from = 11, 16 epochs;
   base_lr == peak_lr gives the batch-256 recipe without warm-up. */
double blstm_lr_schedule(int epoch, double base_lr, double peak_lr, int warmup_epochs, int anneal_from);

/* The alternating ring matching of section 3.2 (0-based): learners 0,2,4,.. are the senders; on even
   steps sender i pairs with i+1, on odd steps with (i-1) mod R.  R must be even and >= 2. */
int adpsgd_ring_partner(int R, int64_t step, int32_t* partner_out);

/* Options.  BLSTM_OPT_RECURRENT_PATH: 0 (default) runs each layer's T recurrent frames in one
   persistent kernel where the shape allows it (mode 1, H one of 128, 256, 512, 1024, grid
   co-resident on the device), 1 forces one launch per frame everywhere. */
#define BLSTM_OPT_RECURRENT_PATH 1
/* BLSTM_OPT_RECURRENT_SYNC (default 1): how the workgroups of a persistent kernel exchange h / dE/da
   between frames.  0: plain accesses ordered by agent-scope release/acquire fences around a counter.
   1: the exchanged tensor is pre-filled with a bf16 NaN pattern no result can take; elements are
   stored write-through at agent scope, and a consumer proceeds once none of the elements it needs
   still holds the pattern (each element is its own ready flag: written once, so any other value is
   final whatever cache answered; elements that still show the pattern are re-read cache-bypassing). */
#define BLSTM_OPT_RECURRENT_SYNC 2
/* BLSTM_OPT_KEEP_WEIGHT_COPIES (default 0): the passes keep two private copies derived from theta in the workspace
   (layer 0's W_x zero-padded to whole tiles, and U_h transposed for the backward recurrence).  0 = both are
   rebuilt in every pass.  1 = they are kept from step to step for as long as blstm_forward / blstm_backward are
   given the same theta pointer and the caller reports every change of the weights it points to (sgd_step,
   adpsgd_mix, sgd_mix_pair, sync_average, a copy) with blstm_weights_changed before the next pass. */
#define BLSTM_OPT_KEEP_WEIGHT_COPIES 3
/* BLSTM_OPT_TEST_ABORT (for tests of the failure path): 1 = the next blstm_forward raises the abort word of the
   persistent kernels itself, as if one of their waits had been abandoned: every later wait returns at once, all
   kernels run to their end, everything they write is NaN, and blstm_device_status reports BLSTM_ERR_HIP. */
#define BLSTM_OPT_TEST_ABORT 4
/* BLSTM_OPT_DEFER_SOFTMAX_WGRAD (default 0): 1 = softmax_xent_fwd_bwd still writes the loss and dz but leaves the W_s
   and b_s slices of grad to the next blstm_backward on this ctx, which computes them together with the other weight
   gradients in its one grouped launch (one by one these products leave part of the device idle).  Until that call, z
   and the workspace must stay as softmax_xent_fwd_bwd left them, and blstm_backward must be given the same grad
   (BLSTM_ERR_DIM otherwise).  A blstm_forward in between drops what was left over.  Same arithmetic, same results.
   softmax_xent_fwd_bwd_noalloc ignores the option. */
#define BLSTM_OPT_DEFER_SOFTMAX_WGRAD 5
int blstm_set_option(blstm_ctx* ctx, int option, int value);
/* The weights behind theta have changed (see BLSTM_OPT_KEEP_WEIGHT_COPIES).  Host-side only, no device work. */
int blstm_weights_changed(blstm_ctx* ctx);

/* The only call that synchronises: waits for `stream`, then reports whether a persistent kernel
   gave up a wait on another workgroup (BLSTM_ERR_HIP; the results of that step are invalid).
   Returns 0 otherwise.  The failure is also visible without this call: a wavefront that gave up a wait,
   and every persistent launch after it until the next blstm_forward that follows a blstm_device_status,
   adds NaN to what it writes, so the loss, the gradient and the updated weights of such a step are NaN. */
int blstm_device_status(blstm_ctx* ctx, void* stream);

/* bf16 <- RNE(master) over n elements (used once, to create the shadow of the initial weights). */
int blstm_shadow_refresh(const float* theta_master, void* theta_bf16, size_t n, void* stream);

/* Per-kernel-class timing with HIP events on the caller's stream.  enable != 0 starts recording
   around every launch (this serialises nothing but adds event overhead); blstm_profile_read
   synchronises the recorded events and returns, for class index k < n_classes, the summed
   milliseconds and launch counts since the last reset.  blstm_profile_name(k) names class k. */
int         blstm_profile_enable(blstm_ctx* ctx, int enable);
int         blstm_profile_read(blstm_ctx* ctx, double* ms_out, int64_t* launches_out, int n_classes);
int         blstm_profile_classes(void);
const char* blstm_profile_name(int k);

/* Text of the last error on this thread ("" if none). */
const char* blstm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
