/*
 * abtrain.h -- C ABI of the MI355X (gfx950) hot path of AB-training (arxiv 2405.01067).
 *
 * The paper carries every dense layer weight W (m x n, out x in) as two thin factors
 *     W = A B,   A = U_k Sigma_k^(1/2)  (m x k),   B = Sigma_k^(1/2) V_k^T  (k x n)     (Eq. 3)
 * trains the factors in independent groups and periodically merges the group copies
 * (Algorithm 1: all-reduce of A and of B, W <- A B, re-decomposition with the rank rule
 * "drop singular values below sigmaCutoff * sigma_max").  This library is that hot path on
 * one GPU: the factored layer's forward and backward, and the merge of G factor copies; beside
 * them the decomposition of a dense weight (ab_factorize), the optimiser step of the group phase
 * (ab_adamw_step), W <- A B (ab_reconstruct) and the factored layer for convolution weights
 * (lr_conv_fwd, lr_conv_bwd).
 *
 * Conventions shared by every entry point
 *   - All matrices are row-major and contiguous (leading dimension = number of columns).
 *   - Unless a parameter is documented as a HOST pointer it is a DEVICE pointer owned by the
 *     caller; the library never allocates, frees or retains caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  lr_linear_fwd,
 *     lr_linear_bwd, lr_linear_bwd_static, lr_linear_fwd_grouped, lr_linear_bwd_grouped, lr_conv_fwd, lr_conv_bwd, ab_adamw_step and ab_reconstruct enqueue work on it
 *     and return without synchronising the host.  Calls that DO block the host:
 *       ab_merge, ab_merge_batched, ab_factorize, ab_factorize_batched: once after uploading
 *         their layer tables, and from the third Jacobi sweep on once per sweep, for the copy of
 *         the convergence flags of the sweep BEFORE the one just enqueued (the host stays one
 *         sweep ahead, so the GPU does not idle meanwhile).  With more than one layer they also
 *         run layer groups on up to three streams of the library's own (default priority),
 *         forked from and joined back into `stream` inside the call.  The stages they enqueue
 *         last (back-projection) may still be running when they return.  Not capturable in a
 *         HIP graph.
 *       ab_merge_info: waits for `stream`.
 *   - `workspace` is caller-owned device scratch of at least the size the matching
 *     *_workspace_bytes() query returns, 256-byte aligned; its contents are undefined
 *     afterwards.  Calls that share a workspace must be stream-ordered.
 *   - Return value: ABT_OK (0) or a negative abt_status.  Nothing is launched when an error
 *     is returned.  The library never throws, aborts or prints.
 *   - `r` below is the paper's k (the retained rank).
 */
#ifndef ABTRAIN_H_
#define ABTRAIN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ABT_OK = 0,
    ABT_EINVAL = -1,     /* NULL where a pointer is required, bad enum, G < 1, tau outside [0,1] ... */
    ABT_ESHAPE = -2,     /* a dimension is non-positive or violates a documented divisibility/limit */
    ABT_EALIGN = -3,     /* a device pointer is not 16-byte aligned (workspace: 256) */
    ABT_EWORKSPACE = -4, /* workspace NULL or smaller than *_workspace_bytes() */
    ABT_EDTYPE = -5,     /* unknown abt_dtype */
    ABT_ENOCONV = -6,    /* reported by ab_merge_info: the Jacobi sweep cap was hit */
    ABT_EHIP = -7,       /* a HIP runtime call failed (launch error, copy error) */
    ABT_ENOMEM = -8,     /* a host-side table of the call could not be allocated */
    ABT_ETOOLARGE = -9   /* lr_linear_bwd_static: the shape needs more than ABT_STATIC_SCRATCH_BYTES */
} abt_status;

typedef enum {
    ABT_F32 = 0,  /* fp32 storage, fp32 accumulate (fp32 MFMA) */
    ABT_BF16 = 1  /* bf16 storage, fp32 accumulate (bf16 MFMA); factor gradients stay fp32 */
} abt_dtype;

/* Human-readable name of a status code (static string, never NULL). */
const char* abt_status_string(int status);

/* ---------------------------------------------------------------------------------------
 * Factored layer, forward (Eq. 3 applied to a batch: y = x W^T with W = A B).
 *
 *     T[M,r] = X[M,n] . B[r,n]^T          Y[M,m] = T[M,r] . A[m,r]^T
 *
 * X, A, B, Y are of type `dt`.  T_save is optional (NULL = T never leaves the chip in the
 * bf16 path); when given it receives T in type `dt` (bf16: T rounded to nearest-even, the
 * same values the second product consumes).
 * Shapes: M >= 1 arbitrary.  ABT_BF16: m, n multiples of 64 and <= 2^20, r a multiple of 32, r <= 384.
 *         ABT_F32: any positive m, n, r.
 * Workspace: lr_linear_fwd_workspace_bytes (0 for ABT_BF16).
 * ------------------------------------------------------------------------------------- */
int lr_linear_fwd(const void* X, const void* A, const void* B, void* Y, void* T_save,
                  int64_t M, int64_t m, int64_t n, int64_t r, int dt,
                  void* workspace, size_t workspace_bytes, void* stream);

size_t lr_linear_fwd_workspace_bytes(int64_t M, int64_t m, int64_t n, int64_t r, int dt);

/* ---------------------------------------------------------------------------------------
 * Factored layer, backward (chain rule through Eq. 3; during the group phase of
 * Algorithm 1 a group trains A or B and the other factor is frozen, hence the NULL skips).
 *
 *     dT[M,r] = dY[M,m] . A[m,r]           dX[M,n] = dT . B[r,n]
 *     dA[m,r] = dY^T . T                   dB[r,n] = dT^T . X
 *
 * dY, X, T, A, B, dX are of type `dt`; dA and dB are always fp32.
 * T: the tensor saved by the forward, or NULL to recompute it from X and B.
 * dX, dA, dB: any may be NULL, that product is then skipped.
 * accumulate != 0 adds into dA / dB instead of overwriting them (gradient accumulation).
 * The reduction over the M rows uses a fixed split and a fixed summation order: two calls on
 * the same inputs give bit-identical results.
 * Shapes as for the forward.  Workspace: lr_linear_bwd_workspace_bytes.
 * ------------------------------------------------------------------------------------- */
int lr_linear_bwd(const void* dY, const void* X, const void* T, const void* A, const void* B,
                  void* dX, float* dA, float* dB,
                  int64_t M, int64_t m, int64_t n, int64_t r, int dt, int accumulate,
                  void* workspace, size_t workspace_bytes, void* stream);

size_t lr_linear_bwd_workspace_bytes(int64_t M, int64_t m, int64_t n, int64_t r, int dt);

/* ---------------------------------------------------------------------------------------
 * lr_linear_bwd for callers that cannot allocate device memory and have no workspace to hand
 * over: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and kernels as lr_linear_bwd, but the workspace is an
 * array of ABT_STATIC_SCRATCH_BYTES inside the library's device code (each GPU the library
 * runs on holds its own copy until the process ends).  The call allocates nothing, on the
 * host or on the device, and frees nothing.
 * A shape for which lr_linear_bwd_workspace_bytes() exceeds ABT_STATIC_SCRATCH_BYTES is
 * rejected with ABT_ETOOLARGE before anything is enqueued.
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap (different
 * streams, different host threads) race on it and give undefined gradients; calls on one
 * stream are safe back to back.  Nothing in the array has to start at zero, and nothing a
 * call leaves there is read by a later one.
 * ------------------------------------------------------------------------------------- */
#define ABT_STATIC_SCRATCH_BYTES (64u << 20)
int lr_linear_bwd_static(const void* dY, const void* X, const void* T, const void* A, const void* B,
                         void* dX, float* dA, float* dB,
                         int64_t M, int64_t m, int64_t n, int64_t r, int dt, int accumulate,
                         void* stream);

/* ---------------------------------------------------------------------------------------
 * The factored layer for G emulated groups at once (Algorithm 1, group training: every group
 * holds its own copy of A and B, sees its own batch and trains A or B; Sec. "Methodology").
 * All groups share the shapes M, m, n, r and the type; `groups` is a HOST array of G <= 8 entries
 * of device pointers with the meaning they have in lr_linear_fwd / lr_linear_bwd:
 *   forward : X, A, B, Y required, T_save optional (all groups or none).
 *   backward: dY, X, A, B required; T optional (NULL = recomputed); dX, dA, dB optional per group
 *             (a group that trains A passes dB = NULL and the other way round).
 * ABT_BF16: the forward is one launch for all groups; the backward is one launch each for the
 * transposes, the dT/dX chain (two if only some groups ask for dX), the factor gradients of all
 * groups and their split reduction.  ABT_F32: the single-group path, group by group.
 * Results per group are those of the single-group calls up to the summation order of dA / dB
 * (the row split depends on the number of tiles in the launch); two grouped calls on the same
 * inputs give bit-identical results.  Workspace: lr_linear_bwd_grouped_workspace_bytes for the
 * backward, lr_linear_fwd_workspace_bytes * G laid end to end for the ABT_F32 forward without T_save.
 * ------------------------------------------------------------------------------------- */
typedef struct abt_lr_group {
    const void* X;      /* [M, n] */
    const void* A;      /* [m, r] */
    const void* B;      /* [r, n] */
    void* Y;            /* forward out [M, m] */
    void* T_save;       /* forward out [M, r], optional */
    const void* dY;     /* backward in [M, m] */
    const void* T;      /* backward in [M, r], optional */
    void* dX;           /* backward out [M, n], optional */
    float* dA;          /* backward out [m, r] fp32, optional */
    float* dB;          /* backward out [r, n] fp32, optional */
} abt_lr_group;
#define ABT_MAX_GROUPS 8

int lr_linear_fwd_grouped(const abt_lr_group* groups, int G,
                          int64_t M, int64_t m, int64_t n, int64_t r, int dt,
                          void* workspace, size_t workspace_bytes, void* stream);
int lr_linear_bwd_grouped(const abt_lr_group* groups, int G,
                          int64_t M, int64_t m, int64_t n, int64_t r, int dt, int accumulate,
                          void* workspace, size_t workspace_bytes, void* stream);
size_t lr_linear_bwd_grouped_workspace_bytes(int G, int64_t M, int64_t m, int64_t n, int64_t r, int dt);

/* ---------------------------------------------------------------------------------------
 * Merge of G group copies of one layer's factors (Algorithm 1: A <- allReduce(A/worldSize),
 * B <- allReduce(B/worldSize), W <- A B; then the AB decomposition of Eq. 3 with the rank
 * rule of Sec. "Methodology": singular values below tau * sigma_max are removed).
 * The G copies live in one GPU's memory; there is no communication.
 *
 *   mode 0 (the paper): Abar = mean_g A_g, Bbar = mean_g B_g, Wbar = Abar Bbar (rank <= k)
 *   mode 1            : Wbar = mean_g (A_g B_g)                              (rank <= G k)
 *   sigma_1 >= sigma_2 >= ... : singular values of Wbar, U, V its singular vectors
 *   k' = k_fixed if k_fixed > 0, else #{ i : sigma_i >= tau * sigma_1 } (compared in fp32,
 *        at least 1), clipped to k_cap and to the number of computed singular values
 *   A_out = U_k' Sigma_k'^(1/2),  B_out = Sigma_k'^(1/2) V_k'^T                   (Eq. 3)
 *
 * A_copies, B_copies: HOST arrays of G device pointers; A_g is m x k, B_g is k x n, fp32.
 *                     The arrays are read before the call returns.
 * tau in [0,1]; k_fixed >= 0.
 * A_out [m, k_cap], B_out [k_cap, n]: fp32; columns (rows) >= k' are zero-filled.
 * S_out [k_cap]: fp32, descending; entries >= the number of computed values are zero.
 * k_out: one int32 in device memory receiving k'.
 * W_out: optional fp32 [m, n] receiving the merged (untruncated) Wbar, the dense weight the
 *        full-rank rebound phase of Algorithm 1 continues from; NULL to skip.
 * Limits: k a multiple of 32; K = k (mode 0) or G k (mode 1) must be <= 2048; 1 <= k_cap.
 * Singular vectors of (near-)zero singular values (sigma_i <= 1e-7 sigma_1) are returned as
 * zero columns/rows: Sigma^(1/2) annihilates them in Eq. 3 anyway.
 * The SVD runs a one-sided Jacobi iteration with a sweep cap (abt_set_jacobi_max_sweeps);
 * ab_merge_info reports sweeps used and whether it converged.
 * ------------------------------------------------------------------------------------- */
int ab_merge(const float* const* A_copies, const float* const* B_copies, int G,
             int64_t m, int64_t n, int64_t k, float tau, int64_t k_fixed, int mode,
             float* A_out, float* B_out, float* S_out, int32_t* k_out, int64_t k_cap,
             float* W_out, void* workspace, size_t workspace_bytes, void* stream);

size_t ab_merge_workspace_bytes(int G, int64_t m, int64_t n, int64_t k, int64_t k_cap, int mode);

/* One layer of a batched merge; fields as the arguments of ab_merge. */
typedef struct {
    const float* const* A_copies; /* HOST array of G device pointers */
    const float* const* B_copies; /* HOST array of G device pointers */
    int32_t G;
    int32_t mode;
    int64_t m, n, k;
    float tau;
    int64_t k_fixed;
    float* A_out;
    float* B_out;
    float* S_out;
    int32_t* k_out;
    int64_t k_cap;
    float* W_out;
} abt_merge_desc;

/* The same merge for L layers at once (one model's layer set per call): every stage is one
 * grouped launch over all layers instead of L launches.  `layers` is a HOST array read
 * before the call returns.  Layers may differ in every field. */
int ab_merge_batched(const abt_merge_desc* layers, int L,
                     void* workspace, size_t workspace_bytes, void* stream);

size_t ab_merge_batched_workspace_bytes(const abt_merge_desc* layers, int L);

/* After the stream work of ab_merge / ab_merge_batched on `workspace` has been enqueued:
 * waits for `stream`, then reports for layer `layer` (0 for ab_merge) the Jacobi sweeps used
 * and the number of singular values computed.  Returns ABT_OK, or ABT_ENOCONV when that
 * layer hit the sweep cap (results were still written), ABT_EINVAL when `layer` is not a layer
 * of the last merge that ran on this workspace.  sweeps / n_sigma: HOST, may be NULL. */
int ab_merge_info(const void* workspace, int layer, int32_t* sweeps, int32_t* n_sigma,
                  void* stream);

/* -------------------------------------------------------------------------------------
 * ab_factorize: Eq. 3 for a DENSE weight, the abDecomposition step of Algorithm 1 that opens
 * every low-rank phase: W [m, n] fp32 -> singular values sigma_1 >= ..., k' by the cut-off
 * rule of ab_merge (tau, k_fixed), A_out = U_k' Sigma_k'^(1/2) [m, k_cap],
 * B_out = Sigma_k'^(1/2) V_k'^T [k_cap, n], S_out [k_cap], k_out (device int32).
 * Where the paper transposes W when n > m, this routine keeps W as it is and factors it
 * trivially as W I (n <= m) or I W (n > m) with the identity on the short side, then runs
 * the pipeline of ab_merge on that pair: K = min(m, n) singular values are computed.
 * Limits: min(m, n) a multiple of 32 and <= 2048.  Outputs, zero-filling, the treatment of
 * numerically zero singular values and stream behaviour as for ab_merge.
 * ab_merge_info applies to the workspace of an ab_factorize / ab_factorize_batched call too.
 * ab_factorize_batched: L dense weights in one call (every stage one grouped launch);
 * `layers` is a HOST array read before the call returns.
 * ------------------------------------------------------------------------------------- */
int ab_factorize(const float* W, int64_t m, int64_t n, float tau, int64_t k_fixed,
                 float* A_out, float* B_out, float* S_out, int32_t* k_out, int64_t k_cap,
                 void* workspace, size_t workspace_bytes, void* stream);

size_t ab_factorize_workspace_bytes(int64_t m, int64_t n, int64_t k_cap);

typedef struct {
    const float* W;               /* [m, n] fp32 */
    int64_t m, n;
    float tau;
    int64_t k_fixed;
    float* A_out;                 /* [m, k_cap] */
    float* B_out;                 /* [k_cap, n] */
    float* S_out;                 /* [k_cap] */
    int32_t* k_out;
    int64_t k_cap;
} abt_factorize_desc;

int ab_factorize_batched(const abt_factorize_desc* layers, int L,
                         void* workspace, size_t workspace_bytes, void* stream);

size_t ab_factorize_batched_workspace_bytes(const abt_factorize_desc* layers, int L);

/* -------------------------------------------------------------------------------------
 * Group-training step (group-training phase of Algorithm 1; Sec. "Learning rate rebound").
 * A group trains one factor of every layer and keeps the other frozen: call lr_linear_bwd
 * with the frozen factor's gradient pointer NULL (its product is skipped), then ab_adamw_step
 * on the trained factors of all layers at once.
 *
 * ab_adamw_step: one step of Adam with decoupled weight decay (the optimiser of the paper's
 * experiments) on n tensors in one launch per 48 tensors.  For every element, in fp32:
 *     m' = beta1 m + (1 - beta1) g            v' = beta2 v + (1 - beta2) g^2
 *     u  = (m' / (1 - beta1^step)) / (sqrt(v' / (1 - beta2^step)) + eps)
 *     theta' = theta - lr * lr_scale * (u + weight_decay * theta)
 * lr_scale is the rebound factor of the step (ab_lr_rebound_scale, or 1).  step >= 1 is the
 * 1-based count of optimiser steps the state has seen including this one.  The
 * hyper-parameters are doubles: 1 - beta, the two bias corrections and lr * lr_scale are
 * evaluated on the host in double precision and each rounded once to fp32 for the kernel.
 * `tensors` is a HOST array read before the call returns.  Per tensor: param, exp_avg,
 * exp_avg_sq (fp32, DEVICE, updated in place), grad (fp32, DEVICE, read only), param_bf16
 * (DEVICE, may be NULL: if given, receives theta' rounded to bf16, the copy the bf16 layer
 * kernels read), count elements (>= 0; 0 skips the tensor).  All pointers 16-byte aligned;
 * tensors must not overlap.  The result is deterministic.  No workspace, no allocation.
 * Errors: ABT_EINVAL (n < 0, NULL table or pointer, step < 1, betas outside [0, 1),
 * eps < 0 or any hyper-parameter not finite), ABT_ESHAPE (count < 0), ABT_EALIGN.
 * ------------------------------------------------------------------------------------- */
typedef struct {
    float* param;
    const float* grad;
    float* exp_avg;
    float* exp_avg_sq;
    void* param_bf16;             /* may be NULL */
    int64_t count;
} abt_adamw_tensor;

int ab_adamw_step(const abt_adamw_tensor* tensors, int n, int64_t step,
                  double lr, double lr_scale, double beta1, double beta2, double eps,
                  double weight_decay, void* stream);

/* Factor applied to the scheduled learning rate i steps (0-based) after the parameters changed
 * shape (Sec. "Learning rate rebound": the rate drops to near zero and climbs back over
 * rebound_steps steps; the climb is taken as linear): min(1, (i + 1) / rebound_steps);
 * 1 when rebound_steps <= 0 or i < 0 is not meaningful (i < 0 is treated as 0).  Host only. */
double ab_lr_rebound_scale(int64_t i, int64_t rebound_steps);

/* W [m, n] = A [m, k] . B [k, n] (fp32, DEVICE, row-major): the hand-off from the averaged
 * factors back to the full-rank weight at the end of a low-rank phase (Algorithm 1).
 * m, n, k >= 1.  Errors: ABT_EINVAL, ABT_ESHAPE, ABT_EALIGN, ABT_EHIP. */
int ab_reconstruct(const float* A, const float* B, float* W,
                   int64_t m, int64_t n, int64_t k, void* stream);

/* -------------------------------------------------------------------------------------
 * Factored convolution (Sec. "Methodology": a weight with more than two dimensions is flattened
 * over its trailing dimensions to give the matrix W of Eq. 3).  A kh x kw convolution weight
 * [m, kh, kw, C] flattened to W [m, kh kw C] = A [m, r] . B [r, kh kw C]: B acts as a kh x kw
 * convolution to r channels, A as a 1 x 1 convolution.  The patch matrix is never materialised:
 * the kernels gather it from the activation.
 * Layout: activation act [N, H, W, C] channels last; the flattened axis of B is tap-major,
 * column (ky kw + kx) C + c.  Zero padding kh/2, kw/2, kh and kw odd, stride 1 or 2 in both
 * directions: output pixel (y', x') is centred on input pixel (stride y', stride x'), the output
 * grid is H' x W' = ceil(H / stride) x ceil(W / stride) (ResNet-50's down-sampling 3 x 3 and 1 x 1
 * convolutions are the stride-2 case).  Y [N H' W', m], T [N H' W', r], dY likewise (row = output
 * pixel, row-major); dAct has act's shape.  bf16 only (fp32 accumulation).
 *   lr_conv_fwd:  T = patches(act) . B^T,  Y = T . A^T          (T_save may be NULL)
 *   lr_conv_bwd:  dT = dY . A,  dA = dY^T . T,  dB = dT^T . patches(act),
 *                 dAct = adjoint of the patch extraction applied to dT . B
 *     dAct [N, H, W, C] bf16, dA [m, r] and dB [r, kh kw C] fp32; each may be NULL (skipped);
 *     T may be NULL (recomputed); accumulate != 0 adds into dA, dB.
 * Limits: C and m multiples of 64; r a multiple of 32, <= 384 and not 224, 288 or 352;
 * kh kw C <= 2^20; N H W < 2^31.  Errors as for lr_linear_*; ABT_EDTYPE for dtype != ABT_BF16.
 * ------------------------------------------------------------------------------------- */
typedef struct {
    int64_t N, H, W, C;
    int32_t kh, kw;
    int32_t stride;               /* 1 or 2 */
    int32_t reserved;             /* 0 */
} abt_conv_geom;

int lr_conv_fwd(const void* act, const void* A, const void* B, void* Y, void* T_save,
                const abt_conv_geom* geom, int64_t m, int64_t r, int dtype, void* stream);

int lr_conv_bwd(const void* dY, const void* act, const void* T, const void* A, const void* B,
                void* dAct, float* dA, float* dB,
                const abt_conv_geom* geom, int64_t m, int64_t r, int dtype, int accumulate,
                void* workspace, size_t workspace_bytes, void* stream);

size_t lr_conv_bwd_workspace_bytes(const abt_conv_geom* geom, int64_t m, int64_t r, int dtype);

/* Work-group height of the bf16 chain kernel (T = X B^T, Y = T A^T and the dT / dX half of the
 * backward): 0 = chosen from the batch size (default), 64 or 128 = forced where the rank allows it.
 * A tuning and test switch; the results do not depend on it beyond fp32 summation order.  Other
 * values are ignored.  Returns the previous setting. */
int abt_set_chain_rows(int rows);

/* Column parts of the 128-row chain kernel: 0 = chosen from the shape (default), 1..8 = forced
 * (capped by the number of 128-column output tiles).  With n parts every row block is served by n
 * work-groups that each repeat the first product and do 1/n of the second.  A tuning and test
 * switch.  Returns the previous setting. */
int abt_set_chain_parts(int parts);

/* Sweep cap of the Jacobi SVD (default 30, clamped to [1, 64]; sweeps stop as soon as every layer
 * has converged: 8 for 384-wide cores with a power-law spectrum, 11 to 15 for 768-wide ones);
 * returns the previous value. */
int abt_set_jacobi_max_sweeps(int max_sweeps);

/* Upper bound on the layer groups of the Jacobi stage of a batched merge (Section "Methodology",
 * the re-decomposition of every layer): the layers of a batch are independent, and the library
 * runs them in up to four groups on streams of its own (default priority, joined back into the
 * caller's stream before the call returns) so that the phases of their rounds overlap.  0 = as
 * many as the library allows (default), 1 = everything on the caller's stream.  A measurement
 * switch; returns the previous setting. */
int abt_set_merge_groups(int groups);

/* Stage timers of ab_merge_batched / ab_factorize_batched (a measurement switch, off by default;
 * returns the previous setting).  While on, a call records HIP events on the caller's stream at
 * its stage boundaries, and ab_merge_stage_ms waits for the last call to finish and writes the
 * elapsed milliseconds of its ABT_MERGE_STAGES stages to the HOST array `ms`, in the order of
 * Algorithm 1's merge followed by Eq. 3:
 *   0 average of the copies + Gram matrices      1 Cholesky factors of the Gram matrices
 *   2 K x K core product                         3 Jacobi sweeps of the core (all layer groups)
 *   4 singular values, rank rule, projectors     5 back-projection A', B' (and W when asked for)
 * Returns ABT_EINVAL if ms is NULL and ABT_EHIP if no timed call has completed. */
#define ABT_MERGE_STAGES 6
int abt_set_merge_stage_timing(int on);
int ab_merge_stage_ms(float* ms);

#ifdef __cplusplus
}
#endif
#endif /* ABTRAIN_H_ */
