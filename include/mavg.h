/*
 * mavg -- model-averaging DNN training hot path for AMD MI355X (gfx950).  C ABI.
 *
 * The operations are those of "Experiments on Parallel Training of Deep Neural Network using Model
 * Averaging" (arXiv 1507.01239): minibatch SGD on a sigmoid/softmax DNN (Sec. 5.1, eq. 3), periodic
 * parameter averaging across model replicas (Sec. 3, eqs. 1-2), RBM pretraining by one-step
 * contrastive divergence (Sec. 5.1) and the natural-gradient preconditioned update (Sec. 4, eqs. 4-5).
 *
 * Conventions (all entry points)
 *   - Every function returns 0 on success or a negative MAVG_E_* code.  Nothing throws or aborts.
 *   - Arguments are validated on the host before anything is launched, so a call that returns
 *     MAVG_E_NULL / _DIM / _ALIGN / _FLAG / _WORKSPACE has not touched the device.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary host
 *     memory read during the call.  The library allocates nothing, frees nothing, keeps no pointer
 *     after the call returns and never synchronises: kernels are enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and the call returns.
 *     Two documented exceptions: dnn_backward_update with MAVG_USE_NGSGD (an internal stream, see there) and
 *     rbm_cd1_step_static (a static device array).
 *   - Matrices are dense row-major float32.  Every device pointer must be 16-byte aligned; replica
 *     strides are counted in elements.
 *   - Workspace: the caller passes a device scratch buffer of at least the size the matching
 *     *_workspace_bytes() query returns; its contents are undefined on entry and exit.
 *   - No floating-point reduction uses atomics (every such sum has one owner and a fixed order), so results are
 *     bitwise reproducible run to run on the same device.  The only atomic is the integer count of
 *     dnn_count_correct, whose result does not depend on the order of the additions.
 *
 * Parameter vector ("theta") of a network with widths d_0..d_L:
 *     [ W_1 | b_1 | W_2 | b_2 | ... | W_L | b_L ],   W_l is d_l x d_{l-1} row-major (row = output unit).
 * Activation buffer ("acts") for a minibatch of n rows:
 *     [ A_1 | A_2 | ... | A_L ],   A_l is n x d_l;  A_l = sigmoid(.) for l < L, A_L = softmax posteriors.
 */
#ifndef MAVG_H
#define MAVG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MAVG_OK            0
#define MAVG_E_NULL       (-1)  /* a required pointer is NULL                                   */
#define MAVG_E_DIM        (-2)  /* a dimension or count is out of range                          */
#define MAVG_E_ALIGN      (-3)  /* a pointer is not 16-byte aligned or a stride is too small     */
#define MAVG_E_FLAG       (-4)  /* unknown flag bit or unsupported mode                          */
#define MAVG_E_LAUNCH     (-5)  /* the HIP runtime reported an error at launch                   */
#define MAVG_E_WORKSPACE  (-6)  /* workspace missing or smaller than *_workspace_bytes()         */

#define MAVG_MAX_LAYERS   64

/* dnn_backward_update flags */
#define MAVG_MEAN_GRAD    1u    /* scale the output error by 1/n (gradient of the mean loss)     */
#define MAVG_USE_NGSGD    2u    /* precondition each layer's gradient factors (needs ng_state)   */
#define MAVG_NG_FIRST     4u    /* with MAVG_USE_NGSGD: first minibatch on freshly initialised
                                   states (each state is folded three times before it is applied) */
#define MAVG_NG_APPLY_ONLY 8u   /* with MAVG_USE_NGSGD: precondition with the states as they are and
                                   leave them unchanged (a caller that folds only every few
                                   minibatches sets it on the others); not together with MAVG_NG_FIRST */

/* ngsgd_precondition `update` modes */
#define MAVG_NG_APPLY        0  /* precondition only                                             */
#define MAVG_NG_UPDATE       1  /* precondition, then fold the minibatch into the state          */
#define MAVG_NG_INIT_UPDATE  2  /* first minibatch on a fresh state: fold three times, then as 1 */

/* rbm_cd1_step */
#define MAVG_VIS_BERNOULLI 0
#define MAVG_VIS_GAUSSIAN  1
#define MAVG_SAMPLE_V1     1u   /* flags bit0: sample the Bernoulli reconstruction               */

/* Hidden-unit nonlinearity (Sec. 5.1 names tanh in one sentence and sigmoids in the next; every benchmarked
   configuration uses the sigmoid). */
#define MAVG_ACT_SIGMOID 0
#define MAVG_ACT_TANH    1

/* Network shape: n_layers affine layers, dims = host array of n_layers+1 widths d_0..d_L (all >= 1);
   hidden_act = MAVG_ACT_* for layers 1..L-1 (the output layer is always a softmax). */
typedef struct {
    int32_t n_layers;
    int32_t hidden_act;
    const int32_t* dims;
} mavg_shape;

/* Version / build identification: returns a static host string. */
const char* mavg_version(void);
/* Text of the last HIP error behind a MAVG_E_LAUNCH on this host thread (static host string). */
const char* mavg_last_error(void);

/* ---- sizes (host only; negative MAVG_E_* on invalid shape) ----------------------------------- */

/* Number of float32 parameters P of the network. */
int64_t mavg_param_count(const mavg_shape* shape);
/* Number of float32 elements of the activation buffer for n rows: n * (d_1 + ... + d_L). */
int64_t mavg_act_count(const mavg_shape* shape, int32_t n);
/* Bytes of workspace dnn_forward / dnn_backward_update need for k replicas of n rows.
   `flags` as for dnn_backward_update; `ng_rank` is the NG-SGD rank (ignored without MAVG_USE_NGSGD). */
int64_t mavg_workspace_bytes(const mavg_shape* shape, int32_t n, int32_t k, uint32_t flags, int32_t ng_rank);

/* ---- DNN forward  (Sec. 5.1: sigmoid hidden layers, softmax output) ---------------------------- */
/*
 * For every replica r in [0,k):  A_0 = x_r;  A_l = sigmoid(A_{l-1} W_l^T + b_l) for l < L;
 * A_L = softmax rows of (A_{L-1} W_L^T + b_L), computed with the row maximum subtracted.
 *   theta  device, replica r at theta + r*theta_stride  (theta_stride >= P, multiple of 4)
 *   x      device, n x d_0, replica r at x + r*x_stride  (x_stride >= n*d_0 or 0 to share one batch)
 *   acts   device, written; replica r at acts + r*act_stride (act_stride >= mavg_act_count, multiple of 4)
 *   n      rows per replica, 1 <= n <= 65534;  1 <= k <= 65535 (MAVG_E_DIM otherwise, here and in dnn_backward_update)
 */
int32_t dnn_forward(const mavg_shape* shape, int32_t k,
                    const float* theta, int64_t theta_stride,
                    const float* x, int64_t x_stride, int32_t n,
                    float* acts, int64_t act_stride,
                    void* workspace, int64_t workspace_bytes, void* stream);

/* ---- DNN backward + SGD update  (eq. 3: theta <- theta + alpha g, g = -d loss / d theta) ------ */
/*
 * Consumes the activations dnn_forward wrote for the same theta, x and n.  For every replica:
 *   delta_L = s (A_L - onehot(labels)),  s = 1/n with MAVG_MEAN_GRAD else 1      (cross-entropy)
 *   for l = L..1:  G_l = delta_l^T A_{l-1},  g_l = column sums of delta_l,
 *                  delta_{l-1} = (delta_l W_l) * A_{l-1} * (1 - A_{l-1})   (with W_l before its update)
 *                  W_l <- W_l - lr G_l,  b_l <- b_l - lr g_l
 * With MAVG_USE_NGSGD the two factors [A_{l-1}, 1] and delta_l are passed through
 * ngsgd_precondition (Sec. 4, eq. 4) before they are multiplied; the delta that is propagated
 * downwards is not.  Every call folds its minibatch into the 2*L states (update mode MAVG_NG_UPDATE;
 * MAVG_NG_INIT_UPDATE with MAVG_NG_FIRST) unless MAVG_NG_APPLY_ONLY is set (mode MAVG_NG_APPLY: the
 * states are read and left as they are).
 * With MAVG_USE_NGSGD (and neither MAVG_NG_FIRST nor MAVG_NG_APPLY_ONLY, at most 16 layers) the folds run on an
 * internal stream beside the weight update: the first such call of a host thread on a device creates one stream
 * (default priority, non-blocking) and three events that live until the process ends; the call forks that stream
 * from `stream` and joins it back before it returns, so everything the call enqueues is complete before anything
 * enqueued on `stream` afterwards starts, and results are bit-identical to the serial order.  Make that first call
 * outside a stream capture.  MAVG_NG_SERIAL_FOLD=1 in the environment (read once per host thread and device) keeps
 * every launch on `stream`.
 *   labels    device int32, n per replica, replica r at labels + r*label_stride (label_stride >= n, or 0 to share
 *             one label vector); each in [0, d_L)
 *             (an out-of-range label contributes no "-1" and no loss; it is not detected)
 *   ng_state  device, required with MAVG_USE_NGSGD: for each replica r, 2*L states laid out as
 *             [in_1, out_1, in_2, out_2, ...], state (r, j) at ng_state + (r*2L + j)*ng_state_stride
 *             bytes; in_l has dim d_{l-1}+1, out_l has dim d_l; every state must hold
 *             ngsgd_state_bytes(max_dim+1, rank) bytes (ng_state_stride >= that, multiple of 16).
 *   loss_sum  device, nullable: k floats; receives sum_n -log A_L[n, label_n] per replica (summed, not
 *             averaged; +inf if a posterior underflowed to 0).
 */
int32_t dnn_backward_update(const mavg_shape* shape, int32_t k,
                            float* theta, int64_t theta_stride,
                            const float* x, int64_t x_stride,
                            const int32_t* labels, int64_t label_stride, int32_t n,
                            const float* acts, int64_t act_stride,
                            float lr, uint32_t flags,
                            void* ng_state, int64_t ng_state_stride, int32_t ng_rank,
                            float ng_alpha, float ng_eta,
                            float* loss_sum,
                            void* workspace, int64_t workspace_bytes, void* stream);

/* ---- model averaging  (Sec. 3, eqs. 1-2; every replica receives the mean, as after an all-reduce) */
/*
 * theta_r[i] <- (1/k) * sum_{j=0..k-1} theta_j[i]   for r in [0,k), i in [0,count).
 * The sum is a balanced pairwise tree in float32, ((t0+t1)+(t2+t3))+((t4+t5)+(t6+t7)) for k = 8 (for k > 8:
 * blocks of 8 replicas, then a tree over the block sums), multiplied once by the float32 value 1/k;
 * for k a power of two, identical replicas are therefore returned bit for bit.
 *   theta  device, replica r at theta + r*theta_stride;  theta_stride >= count, multiple of 4
 *   count  >= 0 (0 is a no-op);  1 <= k <= 64.  Needs no workspace.
 * For k >= 6 the mean is first written to replica 0 and then copied to the others (two streaming passes).
 */
int32_t replicas_average(float* theta, int64_t theta_stride, int64_t count, int32_t k, void* stream);

/* ---- RBM CD-1  (Sec. 5.1: greedy layer-wise RBM pretraining; first RBM has real-valued input) -- */
/*
 * One contrastive-divergence (CD-1) minibatch update, in place:
 *   P_h0 = sigmoid(V0 W^T + c);  H0 = [u < P_h0]  (Philox uniform, phase 0, strict <)
 *   V1   = H0 W + a (Gaussian) | sigmoid(H0 W + a) (Bernoulli) | [u' < sigmoid(H0 W + a)] (Bernoulli,
 *          MAVG_SAMPLE_V1, phase 1);   P_h1 = sigmoid(V1 W^T + c)
 *   dW = (P_h0^T V0 - P_h1^T V1)/n,  da = mean_n(V0 - V1),  dc = mean_n(P_h0 - P_h1)
 *   M <- momentum*M + lr*d;  param <- param + M          recon_err = sum (V0 - V1)^2
 * Uniform of flat element e (row-major index in the n x n_hid or n x n_vis matrix):
 *   word (e & 3) of Philox4x32-10(counter = (e >> 2, step, layer, phase), key = (seed lo32, seed hi32)),
 *   u = (word >> 8) * 2^-24.
 *   w n_hid x n_vis; a n_vis; c n_hid; mw, ma, mc momentum buffers of the same sizes (all device, in place)
 *   v0 device n x n_vis;  recon_err device float, nullable
 * Errors: MAVG_E_NULL, MAVG_E_DIM, MAVG_E_FLAG (unknown vis_type or flag; MAVG_SAMPLE_V1 with Gaussian visibles),
 * MAVG_E_ALIGN, MAVG_E_WORKSPACE, MAVG_E_LAUNCH.
 */
int64_t rbm_workspace_bytes(int32_t n_vis, int32_t n_hid, int32_t n);
int32_t rbm_cd1_step(int32_t n_vis, int32_t n_hid, int32_t vis_type,
                     float* w, float* a, float* c, float* mw, float* ma, float* mc,
                     const float* v0, int32_t n, float lr, float momentum,
                     uint64_t seed, uint32_t step, uint32_t layer, uint32_t flags,
                     float* recon_err, void* workspace, int64_t workspace_bytes, void* stream);
/*
 * Where rbm_cd1_step leaves the intermediate matrices of its last call inside the workspace, for a caller that
 * wants to look at them afterwards (they stay valid until the workspace is used again).  out: host, 8 entries =
 * (byte offset from the workspace pointer rounded up to a multiple of 256, row stride in floats) of
 *   P_h0 (n x n_hid), H0 (n x n_hid, 0.0 / 1.0), V1 (n x n_vis), -P_h1 (n x n_hid, stored negated), in this order.
 * Host only; MAVG_E_NULL / MAVG_E_DIM on invalid arguments.
 */
int32_t rbm_workspace_layout(int32_t n_vis, int32_t n_hid, int32_t n, int64_t* out);
/*
 * rbm_cd1_step for callers that cannot allocate or own no scratch memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same step, same kernels and bit-identical results, with
 * the workspace in a static device array of MAVG_RBM_STATIC_SCRATCH_BYTES inside the library instead of a
 * caller-provided buffer.  Arguments as rbm_cd1_step without workspace / workspace_bytes.
 *   - Size limit: returns MAVG_E_WORKSPACE, before anything is launched, when
 *     rbm_workspace_bytes(n_vis, n_hid, n) - 256 exceeds MAVG_RBM_STATIC_SCRATCH_BYTES
 *     (2048 x 2048 needs 28 MiB at minibatch 512 and fits; 440 x 2048 needs 14.9 MiB at minibatch 256, 36 MiB at 1024).
 *   - Calls no allocator.  The first call on a device looks up that device's address of the array
 *     (hipGetSymbolAddress) and keeps it; make that first call outside a stream capture.
 *   - Each device holds its own copy of the array from module load until the process ends.  All calls on a device
 *     share it and it keeps the last call's contents (nothing in it needs to start at zero: every element a
 *     result depends on is written first).  Calls that overlap on one device, on different streams or from
 *     different threads, race: serialise them, or use rbm_cd1_step with separate workspaces.
 */
#define MAVG_RBM_STATIC_SCRATCH_BYTES ((int64_t)32 << 20)
int32_t rbm_cd1_step_static(int32_t n_vis, int32_t n_hid, int32_t vis_type,
                            float* w, float* a, float* c, float* mw, float* ma, float* mc,
                            const float* v0, int32_t n, float lr, float momentum,
                            uint64_t seed, uint32_t step, uint32_t layer, uint32_t flags,
                            float* recon_err, void* stream);
/*
 * The generator of the sampler by itself (Sec. 5.1 pretraining draws its Bernoulli decisions from it):
 * out[4 i .. 4 i + 3] (device, uint32, 16-byte aligned) <- Philox4x32-10 block of counter
 * (first_block + i mod 2^32, step, layer, phase) under key (seed lo32, seed hi32), for i in [0, nblocks).
 * Errors: MAVG_E_NULL, MAVG_E_DIM (nblocks < 0 or > 2^32), MAVG_E_ALIGN, MAVG_E_LAUNCH.
 */
int32_t mavg_philox_fill(uint32_t* out, int64_t nblocks, uint32_t first_block, uint64_t seed, uint32_t step,
                         uint32_t layer, uint32_t phase, void* stream);
/* hidden probabilities sigmoid(V W^T + c) of a trained RBM (the next RBM's input when stacking). */
int32_t rbm_hidden_prob(int32_t n_vis, int32_t n_hid, const float* w, const float* c,
                        const float* v, int32_t n, float* out,
                        void* workspace, int64_t workspace_bytes, void* stream);

/* ---- DNN initialisation from a pretrained RBM  (Sec. 5.1: the networks are initialised from a stack of RBMs
        trained layer by layer; Sec. 5.3, Table 2 compares it with a random start) --------------------------- */
/*
 * Hidden layer `layer` (1-based) of each of the k replicas takes the RBM's parameters:
 *   W_layer <- w  (device, d_layer x d_{layer-1} row-major, the RBM's n_hid x n_vis matrix),
 *   b_layer <- c  (device, d_layer, the RBM's hidden bias).  The visible bias is not used.
 * theta as in dnn_forward (device, read-write here); w, c are not modified.  Asynchronous on `stream`.
 * Errors: MAVG_E_NULL, MAVG_E_DIM (layer outside 1..n_layers, k < 1), MAVG_E_ALIGN (theta_stride < P), MAVG_E_LAUNCH.
 */
int32_t dnn_init_layer_from_rbm(const mavg_shape* shape, int32_t k, float* theta, int64_t theta_stride,
                                int32_t layer, const float* w, const float* c, void* stream);

/* ---- frame accuracy  (Sec. 5.6: the learning-rate schedule is driven by the frame accuracy on held-out
        data) ------------------------------------------------------------------------------------------- */
/*
 * correct[r] (device, int32[k], overwritten) <- number of rows i < n of replica r whose largest posterior
 * acts_L(i, :) (as left by dnn_forward; lowest class index among equal maxima) is labels[r*label_stride + i].
 * The comparison is made on the float32 posteriors.  acts / act_stride / labels / label_stride as in
 * dnn_backward_update (label_stride 0: all replicas share one label vector).  Asynchronous on `stream`.
 * Errors: MAVG_E_NULL, MAVG_E_DIM, MAVG_E_ALIGN (strides too small for k > 1), MAVG_E_LAUNCH.
 */
int32_t dnn_count_correct(const mavg_shape* shape, int32_t k, const float* acts, int64_t act_stride,
                          const int32_t* labels, int64_t label_stride, int32_t n, int32_t* correct, void* stream);

/* ---- NG-SGD preconditioner  (Sec. 4, eq. 4: theta <- theta + alpha E g, E symmetric positive definite,
        standing for the inverse Fisher matrix of eq. 5, approximated online at low rank) ---------- */
/*
 * State blob (device, caller-owned, 16-byte aligned), for dimension `dim` and rank `rank` < dim:
 *   float  R[rank][ld]  (ld = dim rounded up to a multiple of 4; rows orthonormal)
 *   double d[rank]; double rho; int64 t          -- Fisher estimate F = R^T diag(d) R + rho I
 *   int32 sweeps; int32 unconverged               -- Jacobi sweeps the last fold took; number of folds so far whose
 *                                                    eigen-decomposition used all 14 sweeps without meeting its stop
 *                                                    test (off-diagonal norm <= 1e-13 of the diagonal's): 0 is healthy
 * ngsgd_state_init writes R = [I 0], d = rho = 1e-10, t = 0, sweeps = unconverged = 0.
 *
 * ngsgd_precondition, on x (device, n x dim, row stride ldx >= dim), in place:
 *   update = MAVG_NG_INIT_UPDATE (the caller's first minibatch on a fresh state; the library never reads the
 *   state back to the host, so the caller says so): fold x into the state three times first (t stays 0)
 *   beta = rho (1 + alpha) + alpha sum(d)/dim;  e_i = d_i/(d_i + beta)
 *   H = x R^T;  xh = x - H diag(e) R;  x <- xh * ||x||_F / ||xh||_F
 *   update >= MAVG_NG_UPDATE: fold x in:  J = H^T x;  Y = (eta/n) J + (1-eta)(diag(d) + rho I) R;  Z = Y Y^T = U diag(c) U^T;
 *              R <- diag(c)^-1/2 U^T Y;  rho <- [eta ||x||^2/n + (1-eta)(dim rho + sum d) - sum sqrt c]/(dim - rank);
 *              d <- sqrt(c) - rho;  floors rho >= 1e-10, d_i >= max(1e-10, 5e-4 max d);  t <- t + 1
 * The rank x rank work (Z, its eigen-decomposition, d, rho) is done in float64; the n x dim and
 * rank x dim work in float32.  1 <= rank <= 64, rank < dim, n >= 1.
 */
int64_t ngsgd_state_bytes(int32_t dim, int32_t rank);
int64_t ngsgd_workspace_bytes(int32_t dim, int32_t rank, int32_t n);
int32_t ngsgd_state_init(void* state, int32_t dim, int32_t rank, void* stream);
int32_t ngsgd_precondition(void* state, int32_t dim, int32_t rank,
                           float* x, int64_t ldx, int32_t n, float alpha, float eta, int32_t update,
                           void* workspace, int64_t workspace_bytes, void* stream);

/* ---- the dense contraction all of the above are built from (exported for tests and tuning) -------- */
/*
 * C(m,n) = epilogue( sum_{kk<k} A(m,kk) B(kk,n) ), float32 operands, float32 MFMA accumulation.
 *   a_kc != 0: A(m,kk) = a[m*lda + kk], else a[kk*lda + m];   b_kc != 0: B(kk,n) = b[n*ldb + kk], else b[kk*ldb + n]
 *   C(m,n) = c[m*ldc + n]
 *   epi: 0  C = v            1  C = v + bias[n]          2  C = alpha*sigmoid(v + bias[n])
 *        3  C = v * aux(m,n) * (1 - aux(m,n))            4  C = beta*C + alpha*v
 *   cfg: -1 = choose the kernel, else:
 *        0  64x64 tiles, operands loaded global -> LDS directly when they allow it (16-byte aligned rows, k a
 *           multiple of 16, widths of m/n-contiguous operands multiples of 4), else through registers
 *        1  64x64 tiles, always through registers (guarded loads: any shape and alignment);  2  128x128 likewise
 *        3 / 4 / 5  direct-to-LDS 128x64 / 64x128 / 128x128 tiles;  6  as 0 with a shallower LDS ring
 *        7 / 8  direct-to-LDS 32x64 / 32x32 tiles whose contraction is split four ways inside the workgroup
 *        (3, 4, 5, 7, 8 run as 1 when the operands do not allow direct loads)
 *   splits: 0 = choose how many ways the contraction is split across workgroups (partial sums are combined
 *   in split order by a second kernel), else that many; ignored by 7 and 8.
 * All pointers device.  Results are bitwise reproducible for a given (shape, cfg, splits).
 */
int64_t mavg_gemm_workspace_bytes(int32_t m, int32_t n, int32_t k, int32_t cfg, int32_t splits);
int32_t mavg_gemm(const float* a, int64_t lda, int32_t a_kc, const float* b, int64_t ldb, int32_t b_kc,
                  float* c, int64_t ldc, int32_t m, int32_t n, int32_t k,
                  int32_t epi, const float* bias, const float* aux, int64_t ldaux, float alpha, float beta,
                  int32_t cfg, int32_t splits, void* workspace, int64_t workspace_bytes, void* stream);

/*
 * Several independent contractions C_i = epilogue(A_i B_i) of the same operand layouts in ONE launch (64x64 tiles,
 * unsplit contraction): the form in which dnn_backward_update issues the weight gradients and SGD updates of all
 * layers of a step (eq. 3).  Exported for tests and for timing that launch by itself.
 *   problems  host array of `count` records (1 <= count <= 8), read during the call; all pointers inside device
 *   a_kc, b_kc  as in mavg_gemm, shared by all problems
 *   epi, alpha, beta, bias, aux, ldaux per problem as in mavg_gemm
 *   rowsum_dst (nullable, only with a_kc == 0): rowsum_dst[m] <- rowsum_beta rowsum_dst[m] + rowsum_alpha sum_k A(m,k)
 *   a_pad4 / b_pad4: rows of an m/n-contiguous operand may be read up to the next multiple of 4 columns
 * Errors: MAVG_E_NULL, MAVG_E_DIM, MAVG_E_FLAG, MAVG_E_ALIGN, MAVG_E_LAUNCH.
 */
typedef struct {
    const float* a; int64_t lda;
    const float* b; int64_t ldb;
    float* c; int64_t ldc;
    int32_t m, n, k;
    int32_t epi;
    const float* bias; const float* aux; int64_t ldaux;
    float alpha, beta;
    float* rowsum_dst; float rowsum_alpha, rowsum_beta;
    int32_t a_pad4, b_pad4;
} mavg_gemm_problem;
int32_t mavg_gemm_grouped(const mavg_gemm_problem* problems, int32_t count, int32_t a_kc, int32_t b_kc, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MAVG_H */
