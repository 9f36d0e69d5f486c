/*
 * zgr.h -- C ABI of the client-side ZGR step (zeroth-order optimisation with
 * gradient rectification) for one AMD MI355X (gfx950) GPU.
 *
 * The calls follow the paper's statement of the problem:
 *   - objective and two-point estimator: Sec. 3.2, Eq. (9);
 *   - hybrid perturbation z_h = sqrt(alpha/n) z + sqrt((1-alpha)/m) V z_g: Eq. (10);
 *   - rectified estimator: Eq. (11);
 *   - client procedure (perturb, two forward passes, send one scalar) and
 *     edge-server procedure (regenerate z_h from the seed, update): Algorithm 1;
 *   - in-place application of the perturbation to the local model: Sec. 3.1,
 *     workflow step 5.
 *
 * Conventions
 *   - Every pointer marked DEVICE is device memory of the current HIP device,
 *     owned by the caller, and stays valid for the lifetime of the context.
 *     Pointers marked HOST are host memory.
 *   - The library allocates no device memory: parameters, bases, batch and
 *     workspace all come from the caller.
 *   - All work is enqueued on the HIP stream given to zgr_init.  zgr_step
 *     synchronises that stream once (to read the two losses); the other calls
 *     return after enqueueing unless stated otherwise.
 *   - Every call returns a zgr_status; nothing throws across the boundary.
 *     zgr_last_error gives a human-readable message for the last failure.
 *   - One context per stream; a context is not re-entrant.
 */
#ifndef ZGR_H
#define ZGR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct zgr_ctx zgr_ctx; /* opaque, library-owned host object */

typedef enum {
  ZGR_OK = 0,
  ZGR_ERR_NULL = 1,       /* a required pointer is NULL                              */
  ZGR_ERR_SHAPE = 2,      /* tensor / batch shapes do not fit the model              */
  ZGR_ERR_DTYPE = 3,      /* unknown or mixed storage types                          */
  ZGR_ERR_CONFIG = 4,     /* hyper-parameter out of range                            */
  ZGR_ERR_WORKSPACE = 5,  /* workspace too small or misaligned                       */
  ZGR_ERR_DEVICE = 6,     /* a HIP call failed                                       */
  ZGR_ERR_NONFINITE = 7,  /* a loss is NaN/Inf (parameters are still restored)       */
  ZGR_ERR_STATE = 8       /* call not valid for this context (e.g. no model)         */
} zgr_status;

typedef enum { ZGR_F32 = 0, ZGR_BF16 = 1 } zgr_dtype;

/* Scaling of Eq. (10).  UNIT multiplies it by sqrt(n) so that the mean
 * variance per coordinate is 1, the scale of the non-guided z ~ N(0, I):
 *   a = sqrt(alpha),            b = sqrt((1-alpha) rows / k).
 * PAPER is the equation as printed with n = rows*cols, m = k*cols:
 *   a = sqrt(alpha/(rows cols)), b = sqrt((1-alpha)/(k cols)).                 */
typedef enum { ZGR_SCALE_UNIT = 0, ZGR_SCALE_PAPER = 1 } zgr_scale_mode;

typedef enum { ZGR_ARCH_NONE = -1, ZGR_ARCH_LINEAR_LSQ = 0, ZGR_ARCH_DECODER_LM = 1,
               ZGR_ARCH_ENCODER_CLS = 2 } zgr_arch;

/* Which model weight a tensor is.  2-D weights are [out, in] row-major. */
typedef enum {
  ZGR_ROLE_LSQ_W = 0, ZGR_ROLE_TOK_EMB = 1, ZGR_ROLE_POS_EMB = 2,
  ZGR_ROLE_LN1_G = 3, ZGR_ROLE_LN1_B = 4,
  ZGR_ROLE_WQ = 5, ZGR_ROLE_BQ = 6, ZGR_ROLE_WK = 7, ZGR_ROLE_BK = 8, ZGR_ROLE_WV = 9, ZGR_ROLE_BV = 10,
  ZGR_ROLE_WO = 11, ZGR_ROLE_BO = 12, ZGR_ROLE_LN2_G = 13, ZGR_ROLE_LN2_B = 14,
  ZGR_ROLE_W1 = 15, ZGR_ROLE_B1 = 16, ZGR_ROLE_W2 = 17, ZGR_ROLE_B2 = 18,
  ZGR_ROLE_LNF_G = 19, ZGR_ROLE_LNF_B = 20, ZGR_ROLE_CLS_W = 21, ZGR_ROLE_CLS_B = 22,
  ZGR_ROLE_COUNT = 23
} zgr_role;

/* One parameter tensor of the model W in R^d (Sec. 3.2). */
typedef struct {
  void*        theta;      /* DEVICE, 16-byte aligned, rows*cols elements, row-major, MUTATED IN PLACE */
  int64_t      rows, cols; /* 1-D tensors: rows = 1                                            */
  int32_t      dtype;      /* zgr_dtype; all tensors of a context share one                    */
  uint32_t     tensor_id;  /* < 2^31, unique; enters the Philox counter                        */
  const float* U;          /* DEVICE, rows x ldu fp32, orthonormal columns; NULL => isotropic  */
  int32_t      k, ldu;     /* first k columns of U are used (k <= ldu, k <= rows, k <= 64);
                              a guided tensor needs cols % 4 == 0 (cols % 8 with gauss_bits 16);
                              ranks >= 16 and < 16 may be mixed in one table (two kernels serve them) */
  int32_t      role;       /* zgr_role                                                         */
  int32_t      layer;      /* block index, -1 for tensors outside the blocks                   */
} zgr_tensor;

/* Model whose loss the two forward passes evaluate.  arch = ZGR_ARCH_NONE
 * gives a context that can only perturb/update (the edge server of Algorithm 1).
 * Transformer archs: d_model % n_head == 0, head size in {8, 16, 32, 64}; with
 * bf16 storage d_model and d_ff must be multiples of 64.  Wq, Wk, Wv of a layer
 * must be adjacent in memory in that order (one [3 d, d] matrix), and so must
 * bq, bk, bv.  LINEAR_LSQ: one fp32 tensor ZGR_ROLE_LSQ_W [out, in]; the other
 * fields are ignored.                                                           */
/* The two model families of the paper's experiments (Sec. 4, models and datasets) differ in two textbook choices. */
typedef enum { ZGR_ACT_GELU = 0, ZGR_ACT_RELU = 1 } zgr_act;   /* feed-forward activation: erf-GELU | ReLU */

typedef struct {
  int32_t arch;            /* zgr_arch                                                         */
  int32_t n_layer, d_model, n_head, d_ff, vocab, max_pos, n_class;
  float   ln_eps;
  int32_t act;             /* zgr_act                                                          */
  int32_t post_ln;         /* 0: LayerNorm before each sublayer, final LayerNorm LNF before the head;
                            * 1: LayerNorm after each residual sum, x <- LN(x + sublayer(x)), LNF applied to
                            *    the embeddings, none before the head                           */
} zgr_model;

/* Hyper-parameters of Algorithm 1 ("Require" list). */
typedef struct {
  uint64_t seed;           /* shared random seed s                                             */
  float    eps;            /* perturbation scale epsilon                                       */
  float    alpha;          /* mixing ratio alpha in [0, 1] (weight of the isotropic term)      */
  int32_t  scale_mode;     /* zgr_scale_mode                                                   */
  int32_t  gauss_bits;     /* 32: 4 Gaussians per Philox call; 16: 8 per call                  */
  int32_t  fuse_restore_update; /* 0: zgr_step restores theta, zgr_apply_update updates it (two passes);
                                 * 1: zgr_step's last pass does both at once, theta <- theta + (eps - lr g) Z,
                                 *    with the client's own g of Eq. (11) (single client, weight 1)            */
  float    lr;             /* learning rate eta of the fused last pass; ignored when fuse_restore_update = 0  */
} zgr_config;

/* One mini-batch x_i.  All DEVICE.
 *   DECODER_LM : x = int32 tokens [batch, seq]; y, lengths unused (targets are x shifted by one).
 *   ENCODER_CLS: x = int32 tokens [batch, seq]; y = int32 labels [batch]; lengths = int32 [batch],
 *                keys at positions >= lengths[b] are masked out.
 *   LINEAR_LSQ : x = fp32 X [batch, in]; y = fp32 Y [batch, out]; seq ignored.
 * 1 <= batch <= max_batch; seq <= min(max_seq, max_pos), seq >= 2 for DECODER_LM (a next-token
 * target needs two tokens), seq >= 1 for ENCODER_CLS; lengths[b] in [1, seq].                 */
typedef struct {
  const void*    x;
  const void*    y;
  const int32_t* lengths;
  int32_t        batch, seq;
} zgr_batch;

typedef struct {           /* HOST */
  double loss_plus;        /* L(W + eps z_h; x)                                                */
  double loss_minus;       /* L(W - eps z_h; x)                                                */
  float  g;                /* (L+ - L-) / (2 eps), the scalar of Eq. (11)                      */
} zgr_result;

/* Bytes of DEVICE workspace zgr_init needs for this tensor table (only the
 * shapes, dtype, k of the entries are read; theta and U may be NULL here) and
 * forward passes of up to max_batch x max_seq tokens.  The workspace must be
 * 256-byte aligned.  Returns 0 if the arguments are invalid.                   */
size_t zgr_workspace_bytes(const zgr_model* model, const zgr_tensor* tensors, int32_t n_t,
                           int32_t max_batch, int32_t max_seq);

/* Creates a context over n_t caller-owned tensors.  Copies the tensor table
 * and validates it against the model (every role present once per layer,
 * shapes consistent).  hip_stream is a hipStream_t (NULL = default stream).
 * On failure *out is NULL unless the status is about the table itself, in
 * which case no context is made either; the message is then available from
 * zgr_last_error(NULL).                                                        */
zgr_status zgr_init(zgr_ctx** out, const zgr_model* model, const zgr_tensor* tensors, int32_t n_t,
                    const zgr_config* config, void* workspace, size_t workspace_bytes,
                    int32_t max_batch, int32_t max_seq, void* hip_stream);

/* Guided round: install the basis the cloud sent for one tensor (Algorithm 1,
 * the cloud's broadcast in a guided round); U = NULL or k = 0 makes the tensor
 * isotropic (non-guided round).                                                */
zgr_status zgr_set_basis(zgr_ctx* ctx, int32_t tensor_index, const float* U, int32_t k, int32_t ldu);

/* Guided round with the basis sent compressed (Data Transmission Controller,
 * Sec. 3.4, first equation): Uq holds 4-bit codes, rows x ldq BYTES, element l
 * of a row in byte l/2 (low nibble for even l); the kernels restore
 * U[r][l] = lambda * (code - delta) in fp32 while loading the operand, so no
 * fp32 copy of the basis is ever stored.  Uq is DEVICE memory owned by the
 * caller and must stay valid while installed.  Same shape rules as
 * zgr_set_basis (k <= 64, k <= rows, ldq >= (k+1)/2).  zgr_set_basis on the
 * same tensor replaces it.                                                     */
zgr_status zgr_set_basis_q4(zgr_ctx* ctx, int32_t tensor_index, const uint8_t* Uq, int32_t k, int32_t ldq,
                            float lambda, float delta);

/* System-level Pipeline Controller (Sec. 3.3), client side: the basis of this
 * tensor stays in HOST memory (where the link from the cloud delivers it) and
 * is brought to the device layer by layer during every perturbation pass.
 * Tensors with the same `layer` travel together, and consecutive layers are
 * packed into one stage until the stage is large enough to keep the chip busy
 * (8192 tiles of 128 x 128 elements: three layers at d = 2048, every layer its
 * own stage on larger models): the kernel launch that perturbs stage s also
 * reads the bases of stage s + 1 out of host memory into the other of two
 * staging slots in the workspace, so the transfer runs under the arithmetic of
 * stage s and only two stages' bases are ever resident.
 * bits = 32: U_host is fp32 [rows, k]; bits = 4: U_host holds the 4-bit codes
 * of zgr_set_basis_q4, [rows, (k+1)/2 bytes], with their lambda and delta
 * (ignored for bits = 32).  Rows are compact (no row stride).  U_host is owned
 * by the caller, must be PINNED host memory the device can read
 * (hipHostMalloc), 16-byte aligned, and stay valid and unchanged while
 * installed.  Bases of one layer that lie in one host allocation in tensor-table
 * order, each padded to a multiple of 256 bytes, are fetched as one piece.  At
 * most 16 pieces per stage (a layer with more closes the stage early), at most
 * 16 streamed tensors per layer.  The staging slots are sized by
 * zgr_workspace_bytes from the ranks k of the tensor table given to it: a layer
 * whose bases need more is refused with ZGR_ERR_WORKSPACE.  Results are
 * identical to a resident basis.  zgr_set_basis / zgr_set_basis_q4 on the same
 * tensor undo it.                                                              */
zgr_status zgr_set_basis_host(zgr_ctx* ctx, int32_t tensor_index, const void* U_host, int32_t k,
                              int32_t bits, float lambda, float delta);

/* The cloud's side of the same equation, on the device: codes
 * round(U/lambda + delta) clipped to [0, 15] with lambda = (max - min) / 15 and
 * delta = round(-min / lambda) over the first k columns of U [rows, ldu]
 * (fp32 arithmetic, round to nearest even; the zero point as printed in the
 * paper is not a code, this is the reading that maps min to code 0).  U, Uq
 * (rows x ldq bytes) and minmax_dev (2 floats of scratch) are DEVICE memory;
 * lambda_out, delta_out are HOST.  Synchronises the stream once.                */
zgr_status zgr_quantize_basis(const float* U, int64_t rows, int32_t k, int32_t ldu, uint8_t* Uq, int32_t ldq,
                              float* minmax_dev, float* lambda_out, float* delta_out, void* hip_stream);

/* Sec. 3.4, the latency relations that close the section (host arithmetic only,
 * no device work): the smallest share omega in [0, 1] of a layer's guided data
 * of data_bytes bytes that has to travel compressed (to theta of its size,
 * 0 < theta < 1) over a link of bandwidth_bytes_per_s so that the transfer
 * hides under the client's work,
 *     data_bytes (1 - omega (1 - theta)) / bandwidth <= t_cc_s + restore_s_per_byte data_bytes omega
 * (t_cc_s: the client's perturbation time for that layer; restore_s_per_byte:
 * measured cost of restoring compressed data, 0 when the restore is fused into
 * the pass).  The paper prints the left side without the factor in omega; the
 * transfer time of partly compressed data is the reading taken.  *hidden = 1 if
 * the relation holds at *omega, 0 if even omega = 1 does not reach it (then
 * *omega = 1).  ZGR_ERR_CONFIG for non-positive sizes or theta outside (0, 1). */
zgr_status zgr_dtc_omega(double data_bytes, double bandwidth_bytes_per_s, double t_cc_s, double restore_s_per_byte, double theta,
                         double* omega, int32_t* hidden);

/* Same section, the memory relation: client memory in units of the model's own
 * size with the layer pipeline, (1 + 2 / n_layers), less omega (1 - theta) / n_layers
 * when a share omega travels and is held compressed.  HOST arithmetic.        */
zgr_status zgr_dtc_memory_factor(int32_t n_layers, double omega, double theta, double* factor);

/* ---- cloud block of Algorithm 1 (back-propagation on the public dataset, whose gradients build the basis;
 * Sec. 3.2, paragraph on guided perturbation sampling on the cloud) ---- */
/* The basis U [rows, k] (row stride ldu >= k, DEVICE, orthonormal columns) of one weight matrix from n_snap stored
 * gradient snapshots of it (snapshots: HOST array of n_snap DEVICE pointers, each fp32 [rows, cols] row-major): the
 * k-dimensional subspace of R^rows that captures the most of them, i.e. the span of the k leading left singular
 * vectors of [G_1 | ... | G_s] (the paper asks for an orthonormal basis of the gradients' subspace and does
 * not say how a rank is chosen; this is the reading for a basis that acts on every column of the matrix).  Reached by
 * n_iter sweeps of block subspace iteration Q <- orth(sum_t G_t G_t^T Q) from Q = orth(sum_t G_t omega), omega
 * [cols, k] DEVICE fp32 being the caller's seeded standard-normal start; the subspace converges like
 * (sigma_{k+1} / sigma_k)^(2 n_iter).  Only the subspace is defined: compare projectors U U^T.  A column the
 * snapshots do not span (rank below k) comes out as zeros; *dependent_out (HOST, may be NULL; reading it
 * synchronises the stream) counts them.  workspace: DEVICE, 256-byte aligned, zgr_cloud_basis_workspace bytes.   */
size_t     zgr_cloud_basis_workspace(int64_t rows, int64_t cols, int32_t k);
zgr_status zgr_cloud_basis(const float* const* snapshots, int32_t n_snap, int64_t rows, int64_t cols, int32_t k, const float* omega, int32_t n_iter,
                           float* U, int32_t ldu, int32_t* dependent_out, void* workspace, size_t workspace_bytes, void* hip_stream);
/* The cloud's gradient for the least-squares model: G [n_out, n_in] = (X W^T - Y)^T X / batch, all DEVICE fp32 row-major;
 * workspace: DEVICE, batch * n_out floats.  Asynchronous.                                                            */
zgr_status zgr_cloud_lsq_gradient(const float* W, const float* X, const float* Y, int32_t batch, int32_t n_out, int32_t n_in, float* G,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);
/* The cloud's backward pass over the context's model (the back-propagation step of the cloud block of
 * Algorithm 1): *loss_out (HOST) = L(theta; batch) as zgr_loss defines it, and grads[i] (HOST array of n_grads = n_t
 * DEVICE pointers, caller-owned, each rows_i * cols_i fp32 row-major, overwritten) = dL/dtheta_i for every tensor the
 * context was created with, in fp32 whatever the storage type; theta itself is left untouched.  The forward half runs
 * the client's own kernels (so a bf16 model's intermediate results are bf16-rounded exactly as in zgr_loss, except
 * that the activation is evaluated from the fp32 pre-activation, GELU by its erf form) and keeps every layer's results
 * in `workspace` (DEVICE, 256-byte aligned, zgr_cloud_backward_workspace(ctx, batch, seq) bytes: it grows with
 * n_layer * batch * seq * (d_model + d_ff)); both activations and both LayerNorm placements of zgr_model are covered.
 * The backward half is deterministic (no atomics).  Runs on the context's stream and returns after it has finished.
 * seq <= 2048, batch * n_head <= 65535.  Errors: ZGR_ERR_NULL, ZGR_ERR_SHAPE (batch outside the context's limits,
 * n_grads != n_t, seq too long, too many heads), ZGR_ERR_WORKSPACE, ZGR_ERR_STATE (a context without a model),
 * ZGR_ERR_NONFINITE (gradients are then undefined), ZGR_ERR_DEVICE.                                            */
size_t     zgr_cloud_backward_workspace(const zgr_ctx* ctx, int32_t batch, int32_t seq);
zgr_status zgr_cloud_backward(zgr_ctx* ctx, const zgr_batch* batch, float* const* grads, int32_t n_grads, double* loss_out,
                              void* workspace, size_t workspace_bytes);

/* Client block of Algorithm 1 for round/step `step` (< 2^32): perturb all
 * tensors in place by +eps Z, evaluate L+, by -2 eps Z, evaluate L-, restore by
 * +eps Z, Z regenerated from (seed, step) in each pass.  Fills *out.  On
 * return the parameters hold their pre-step values up to rounding of the
 * storage type.  ZGR_ERR_NONFINITE still restores the parameters.
 * With config.fuse_restore_update = 1 the last pass adds (eps - lr g) Z instead
 * (both products in fp32: c = fl(eps - fl(lr g))), which leaves the parameters
 * updated as restore + zgr_apply_update(step, g, lr) would, with one rounding
 * of the storage type fewer; zgr_apply_update must then not be called for this
 * step.  A non-finite loss still restores (adds eps Z) and updates nothing.
 * ZGR_ERR_DEVICE (a launch or copy failed part-way) is the one status after
 * which the parameters are undefined: some tensors may hold a perturbed value. */
zgr_status zgr_step(zgr_ctx* ctx, uint64_t step, const zgr_batch* batch, zgr_result* out);

/* Edge-server block of Algorithm 1 for one client with weight 1:
 * theta <- theta - lr g Z(seed, step).  A pure function of (theta, seed, step,
 * bases, lr*g): valid on a context that never ran the forward passes.  The
 * product lr*g is formed in fp32.  Asynchronous.                                */
zgr_status zgr_apply_update(zgr_ctx* ctx, uint64_t step, float g, float lr);

/* Edge-server block of Algorithm 1 with its sum over local steps t (and over
 * clients, whose weights w_i the caller folds into g):
 *   theta <- theta - lr * sum_q g[q] Z(seed, steps[q]),   q = 0 .. n-1,
 * in ONE read-modify-write pass over the parameters per group of ZGR_MAX_BATCH
 * perturbations (n may exceed it; n = 0 is a no-op): every Z(seed, steps[q]) is
 * regenerated from the seed, the sum is accumulated in fp32 in list order and
 * the result is rounded to the storage type once per pass.  For n > ZGR_MAX_BATCH
 * the call is DEFINED as successive passes over the groups q = 0..7, 8..15, ...
 * in list order, each group one exact-sum-then-round update of the parameters the
 * previous group left (so it equals the same call made group by group, not one
 * rounding of the whole sum).  steps, g: HOST
 * arrays of n entries, steps[q] < 2^32; each product lr*g[q] is formed in fp32.
 * The bases must be those of the steps named (one guidance interval).
 * Asynchronous.  n = 1 equals zgr_apply_update.                                */
#define ZGR_MAX_BATCH 8
zgr_status zgr_apply_updates(zgr_ctx* ctx, int32_t n, const uint64_t* steps, const float* g, float lr);

/* theta <- theta + c Z(seed, step) for all tensors: the single pass that
 * zgr_step and zgr_apply_update are made of.  Asynchronous.                    */
zgr_status zgr_perturb(zgr_ctx* ctx, uint64_t step, float c);

/* One loss evaluation at the current parameters (synchronises the stream). */
zgr_status zgr_loss(zgr_ctx* ctx, const zgr_batch* batch, double* loss_out /* HOST */);

/* zgr_loss of the least-squares model for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): no context, no workspace;
 * the predictions X W^T and the per-example losses live in a static device array of the library (1 MiB + 16 KiB
 * per GPU, held until the process ends).  W [n_out, n_in], X [batch, n_in], Y [batch, n_out]: DEVICE fp32, row-major;
 * loss_out: DEVICE, one double, = ||X W^T - Y||_F^2 / (2 batch) exactly as zgr_loss computes it (same kernels, same
 * order).  Limits: batch <= 4096 and batch * n_out <= 262144; larger sizes return ZGR_ERR_WORKSPACE and launch
 * nothing.  Asynchronous on hip_stream: no synchronisation, no copy to the host, no allocation of any kind.  All
 * calls on one GPU share the one array: calls that overlap on a GPU (different streams or threads) race; calls
 * on one stream are ordered.  Nothing in the array has to be cleared between calls: each call writes every word
 * it later reads.                                                                                             */
zgr_status zgr_lsq_loss_static(const float* W, const float* X, const float* Y, int32_t batch, int32_t n_out, int32_t n_in,
                               double* loss_out /* DEVICE */, void* hip_stream);

void        zgr_destroy(zgr_ctx* ctx);
const char* zgr_last_error(const zgr_ctx* ctx); /* ctx may be NULL: last error of a failed zgr_init */

/* ---- profiling: HIP-event timing of kernel classes on the context's stream ---- */
typedef enum { ZGR_K_PERTURB_TILE = 0 /* guided matrices */, ZGR_K_PERTURB_FLAT = 1 /* isotropic tensors */,
               ZGR_K_GEMM = 2, ZGR_K_ATTN = 3, ZGR_K_NORM = 4, ZGR_K_EMBED = 5, ZGR_K_LOSS = 6,
               ZGR_K_COUNT = 7 } zgr_kernel_class;
/* Enables (1) / disables (0) event recording around every launch and clears the totals. */
zgr_status zgr_profile_enable(zgr_ctx* ctx, int32_t on);
/* Suspends (1) / resumes (0) event recording without clearing the totals or synchronising: lets a caller
 * time a sample of its steps, since two event records per launch are not free.                          */
zgr_status zgr_profile_pause(zgr_ctx* ctx, int32_t paused);
/* Synchronises the stream and returns accumulated milliseconds and launch
 * counts per zgr_kernel_class since zgr_profile_enable (HOST arrays of ZGR_K_COUNT). */
zgr_status zgr_profile_read(zgr_ctx* ctx, double* ms, int64_t* launches);

/* ---- test-only exports: materialise what the fused kernel never stores ---- */
/* Philox4x32-10 of n counters ON THE DEVICE.  ctr: DEVICE u32 [n,4]; key: HOST u32 [2]; out: DEVICE u32 [n,4]. */
zgr_status zgr_debug_philox(const uint32_t* ctr, const uint32_t* key, uint32_t* out, int64_t n, void* hip_stream);
/* Gaussians of flat elements [first, first+n) of one stream: out DEVICE fp32 [n]. */
zgr_status zgr_debug_gauss(uint64_t seed, uint64_t step, uint32_t tensor_id, int32_t stream, int32_t gauss_bits,
                           int64_t first, int64_t n, float* out, void* hip_stream);
/* Z of one tensor as fp32 [rows, cols] (DEVICE), computed by the same code path as the in-place pass. */
zgr_status zgr_debug_fill_z(zgr_ctx* ctx, int32_t tensor_index, uint64_t step, float* Z);
/* Stage size of the layer pipeline of zgr_set_basis_host: consecutive layers share a stage (one launch, one
 * staging slot) until it holds min_tiles tiles of 128 x 128 (x 256 with gauss_bits 16) elements; default 8192,
 * 1 gives one stage per layer.  For tests that want many stages on small models.                          */
zgr_status zgr_debug_set_stage_tiles(zgr_ctx* ctx, int64_t min_tiles);
/* Per-example losses of the last forward (DEVICE -> HOST copy, synchronises):
 * LM: [batch*(seq-1)] token losses; CLS: [batch]; LSQ: [batch].  n must match. */
zgr_status zgr_debug_last_row_losses(zgr_ctx* ctx, float* out /* HOST */, int64_t n);
/* The same for either forward of the last zgr_step: which = 0 the rows of L+, 1 the rows of L-. */
zgr_status zgr_debug_step_row_losses(zgr_ctx* ctx, int32_t which, float* out /* HOST */, int64_t n);
/* Radius sqrt(-2 ln u) for all 2^23 (bits=32) or 2^16 (bits=16) values of the radius uniform, and
 * (cos, sin)(2 pi v) for all 2^24 / 2^16 angle uniforms, as the fused kernel evaluates them. */
zgr_status zgr_debug_radius_table(int32_t gauss_bits, float* out /* DEVICE */, void* hip_stream);
zgr_status zgr_debug_cossin_table(int32_t gauss_bits, float* cos_out, float* sin_out /* DEVICE */, void* hip_stream);

/* One linear layer of the forward pass as the library runs it: out = epilogue(A[M,K] W[N,K]^T + bias),
 * all DEVICE.  dtype: storage type of A, W, bias (bf16 needs K % 64 == 0).  epilogue: 0 store (storage
 * type), 1 GELU then store, 2 add into fp32 out, 3 store fp32.  bias may be NULL.                       */
zgr_status zgr_debug_gemm(int32_t dtype, const void* A, const void* W, const void* bias, void* out, int32_t epilogue,
                          int32_t M, int32_t N, int32_t K, void* hip_stream);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16) by a simple kernel: the known-size
 * reference that hardware traffic counters are calibrated against.                                      */
zgr_status zgr_debug_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* ---- machine ceilings the perturbation pass is rated against (measurement only) ---- */
/* The bare in-place stream buf[i] <- rnd(buf[i] + c) over `bytes` bytes of dtype data in 16-byte vectors, with a
 * grid of `blocks` blocks of 256 threads striding over the buffer: mode 0 read-modify-write, 1 read only, 2 write
 * only.  sink16: 16 bytes of DEVICE memory (written only if the data xor to one particular value).            */
zgr_status zgr_debug_rmw(void* buf, size_t bytes, int32_t dtype, float c, int32_t mode, int32_t blocks, void* sink16, void* hip_stream);
/* Issue rate of one kind of vector instruction: `blocks` blocks of 4 waves each run iters x 64 instructions of
 * kind op (0 v_fma_f32, 1 v_xor_b32, 2 v_bitop3_b32, 3 v_mad_u64_u32, 4 v_mul_hi_u32, 5 v_mul_lo_u32, 6 v_cvt_f32_u32,
 * 7 v_rsq_f32, 8 v_add_u32, 9 v_lshrrev_b32, 10 v_cndmask_b32, 11 v_mul_f32, 12 v_add_f32, 13 v_log_f32,
 * 14 v_cvt_pk_bf16_f32, 15 v_sqrt_f32, 16 v_mov_b32, 17 the matrix-core instruction v_mfma_f32_32x32x16_bf16 on random
 * bf16 register operands, 32768 flops each, 18 v_mfma_f32_32x32x2_f32 on random fp32 register operands, 4096 flops
 * each) in ilp (1, 2 or 4) independent dependent-chains.  out: DEVICE,
 * 4 uint64 per wave (4 * blocks waves): shader cycles of the wave's own run, the 100 MHz real-time counter at its
 * start and at its end, a checksum.  The waves of a SIMD do not advance in step: rates come from the span over all
 * waves (first start to last end).                                                                            */
zgr_status zgr_debug_issue_rate(int32_t op, int32_t ilp, int32_t blocks, int32_t iters, uint64_t* out, void* hip_stream);
/* The same for the Gaussian generator's own parts, with nothing else in the kernel: part 0 one Philox4x32-10 call,
 * 1 two radii sqrt(-2 ln u), 2 two (cos, sin) pairs, 3 two Box-Muller pairs, 4 the whole generator of four
 * Gaussians (one Philox call + two pairs), 5 the two table look-ups alone; iters calls per lane.  out as above. */
zgr_status zgr_debug_generator_rate(int32_t part, int32_t blocks, int32_t iters, uint64_t* out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ZGR_H */
