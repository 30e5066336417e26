/*
 * pufferfish.h -- C ABI of the MI355X (gfx950) library for Pufferfish's
 * pre-factorized low-rank layers: forward and backward of a dense weight W
 * replaced by rank-r factors U V^T.
 *
 * General rules
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The layer
 *     entry points never allocate, free or synchronise; work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream).
 *     The one exception is the benchmark-only pf_timing_* group at the end of
 *     this file, which creates HIP events while enabled and waits for them in
 *     pf_timing_collect(); with timing disabled (the default) nothing of the
 *     kind happens.
 *   - Descriptors are small HOST structs passed by pointer.
 *   - Arrays are dense row-major, last index fastest.
 *   - `dtype` PF_F32: all tensors float.  PF_BF16: activations and factors are
 *     bfloat16, products accumulate in float, activation outputs (Y, dX, T_save)
 *     are rounded to bfloat16.  Parameter gradients (dU, dV, dbias, ...) are
 *     ALWAYS float: descriptors that carry a `wgrad_dtype` accept PF_F32 only.
 *   - Activations, factors, biases and saved tensors must be 16-byte aligned
 *     (any device allocation is); parameter-gradient outputs need only 4-byte
 *     alignment, so they may be slices of ONE flat float buffer laid out back
 *     to back -- the single all-reduce payload of the paper's Section 4
 *     ("implementation details").  Otherwise PF_ERR_UNSUPPORTED.
 *   - `accumulate` != 0 adds parameter gradients to what the buffers hold
 *     (gradient accumulation, back-propagation through time); 0 overwrites.
 *   - Scratch memory comes from the caller: ask pf_*_workspace_bytes(desc),
 *     pass at least that many bytes, 256-byte aligned (PF_ERR_UNSUPPORTED
 *     otherwise).  A NULL workspace is accepted when the query returns 0.
 *     The queries return 0 also for a descriptor the entry point would
 *     reject; the entry point then reports why.
 *   - Every call returns a pf_status.  Arguments are validated on the host
 *     before anything is launched: PF_ERR_NULL (a required pointer is NULL),
 *     PF_ERR_SHAPE (a dimension is not positive, or a convolution has no
 *     output pixel), PF_ERR_UNSUPPORTED (dtype/layout/groups value not built),
 *     PF_ERR_WORKSPACE (workspace too small or NULL), PF_ERR_LAUNCH (HIP
 *     reported an error; see pf_last_hip_error()).  A batch of zero rows
 *     (M, N or B equal to 0) is legal: activation outputs are empty and
 *     non-accumulated parameter gradients are set to zero.
 */
#ifndef PUFFERFISH_H
#define PUFFERFISH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PF_OK = 0,
    PF_ERR_NULL = 1,
    PF_ERR_SHAPE = 2,
    PF_ERR_UNSUPPORTED = 3,
    PF_ERR_WORKSPACE = 4,
    PF_ERR_LAUNCH = 5
} pf_status;

typedef enum { PF_F32 = 0, PF_BF16 = 1 } pf_dtype;
/* Activation layouts of the convolution entry points (only NCHW is built). */
typedef enum { PF_NCHW = 0, PF_NHWC = 1 } pf_layout;

const char *pf_status_string(int status);
/* hipError_t of the last failed launch on the calling thread (0 = none). */
int pf_last_hip_error(void);
/* Library version, major * 100 + minor. */
int pf_version(void);

/* ------------------------------------------------------------------ */
/* Fully connected layer (paper Section 2.1; Appendix B "FC layer";     */
/* Transformer projections and FFN matrices of Section 2.4 are this     */
/* layer with M = number of tokens).                                   */
/*   X[M x in], V[in x r] input-side factor, U[out x r] output-side     */
/*   factor, W = U V^T (out x in), T = X V (M x r), Y = T U^T + bias.   */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t M, in, out, r;
    int dtype;       /* pf_dtype */
    int wgrad_dtype; /* pf_dtype of dU, dV, dbias: PF_F32 (anything else: PF_ERR_UNSUPPORTED) */
    int has_bias;    /* bias[out] is read (fwd) / dbias[out] is written (bwd) */
} pf_linear_desc;

size_t pf_lowrank_linear_fwd_workspace_bytes(const pf_linear_desc *d);
size_t pf_lowrank_linear_bwd_workspace_bytes(const pf_linear_desc *d);

/* Y = (X V) U^T + bias.  T_save (nullable, [M x r], dtype) receives T for
 * the backward pass; when NULL, T never leaves the chip. */
int pf_lowrank_linear_fwd(const pf_linear_desc *d, const void *X, const void *V,
                          const void *U, const void *bias /* nullable */,
                          void *Y, void *T_save /* nullable */,
                          void *workspace, size_t workspace_bytes, void *stream);

/* Given dY[M x out]:  dT = dY U,  dX = dT V^T,  dU = dY^T T,  dV = X^T dT,
 * dbias = column sums of dY.  T_saved (nullable) is the forward pass's
 * T_save; when NULL, T is recomputed from X and V.  dX, dU, dV, dbias are
 * each nullable (skipped); dU, dV, dbias are float. */
int pf_lowrank_linear_bwd(const pf_linear_desc *d, const void *X, const void *V,
                          const void *U, const void *dY,
                          const void *T_saved /* nullable */,
                          void *dX, void *dU, void *dV, void *dbias,
                          int accumulate, void *workspace,
                          size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory or hand over a         */
/* workspace (code running under HIP graph capture, tight serving        */
/* loops, harnesses that forbid hipMalloc): pf_lowrank_linear_bwd with   */
/* its scratch memory in a device array that is part of the library,     */
/* PF_STATIC_SCRATCH_BYTES per GPU, held until the process ends.  Same   */
/* arguments, results and errors as pf_lowrank_linear_bwd minus the      */
/* workspace; a descriptor whose pf_lowrank_linear_bwd_workspace_bytes   */
/* exceeds PF_STATIC_SCRATCH_BYTES gets PF_ERR_WORKSPACE.  The call      */
/* allocates and frees nothing.  All calls on one GPU share that GPU's   */
/* array: calls enqueued on one stream are ordered and safe, calls that  */
/* can overlap on one GPU (different streams, different threads) race.   */
#define PF_STATIC_SCRATCH_BYTES (40u << 20)
size_t pf_static_scratch_bytes(void);
int pf_lowrank_linear_bwd_static(const pf_linear_desc *d, const void *X,
                                 const void *V, const void *U, const void *dY,
                                 const void *T_saved /* nullable */, void *dX,
                                 void *dU, void *dV, void *dbias,
                                 int accumulate, void *stream);

/* ------------------------------------------------------------------ */
/* Several factorized projections of the same shape that read the SAME */
/* input, e.g. the query, key and value matrices of an attention block  */
/* (paper Section 2.4; each is the layer of Section 2.1):              */
/*   Y_g = (X V_g) U_g^T + bias_g,  g = 0 .. groups-1.                  */
/*   V[groups, in, r], U[groups, out, r], bias[groups, out],            */
/*   Y[groups, M, out], T_save[groups, M, r] (nullable).                */
/* Backward: dY[groups, M, out] gives dX = sum_g dY_g U_g V_g^T (ONE    */
/* tensor [M, in]: the input is shared) and dU, dV, dbias per group in  */
/* the layouts of U, V, bias (float; each nullable).  Results equal     */
/* those of `groups` calls of pf_lowrank_linear_fwd/bwd with the input   */
/* gradients added up; X and the running sum dX are read and written    */
/* once instead of once per projection.                                 */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t M, n_in, n_out, r;
    int groups; /* 1 .. 64 */
    int dtype;  /* pf_dtype */
    int has_bias;
} pf_linear_shared_desc;

size_t pf_lowrank_linear_shared_fwd_workspace_bytes(const pf_linear_shared_desc *d);
size_t pf_lowrank_linear_shared_bwd_workspace_bytes(const pf_linear_shared_desc *d);

int pf_lowrank_linear_shared_fwd(const pf_linear_shared_desc *d, const void *X,
                                 const void *V, const void *U,
                                 const void *bias /* nullable */, void *Y,
                                 void *T_save /* nullable */, void *workspace,
                                 size_t workspace_bytes, void *stream);

int pf_lowrank_linear_shared_bwd(const pf_linear_shared_desc *d, const void *X,
                                 const void *V, const void *U, const void *dY,
                                 const void *T_saved /* nullable */, void *dX,
                                 void *dU, void *dV, void *dbias, int accumulate,
                                 void *workspace, size_t workspace_bytes,
                                 void *stream);

/* ------------------------------------------------------------------ */
/* Convolution layer (paper Section 2.2 "Factorizing a convolution      */
/* layer"; Appendix B "Convolution layer").                            */
/*   X[N,Cin,H,W] (NCHW); Uk[r,Cin,k,k] = the r thin k x k basis        */
/*   filters (conv_u; stride and zero padding of the original layer);   */
/*   Vp[Cout,r] = the 1x1 convolution (conv_v; stride 1, no padding);   */
/*   T[N,r,Ho,Wo]; Y[N,Cout,Ho,Wo]; Ho = (H + 2 pad - k) / stride + 1.   */
/*   Cross-correlation (no kernel flip); nothing between the stages.    */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t N, Cin, H, W, Cout, r;
    int k, stride, pad;
    int layout;      /* pf_layout of X, T, Y and their gradients: PF_NCHW (anything else: PF_ERR_UNSUPPORTED) */
    int dtype;       /* pf_dtype */
    int wgrad_dtype; /* pf_dtype of dUk, dVp: PF_F32 (anything else: PF_ERR_UNSUPPORTED) */
} pf_conv_desc;

size_t pf_lowrank_conv_fwd_workspace_bytes(const pf_conv_desc *d);
size_t pf_lowrank_conv_bwd_workspace_bytes(const pf_conv_desc *d);

/* Bytes of the optional W_save buffer: both factors re-ordered the way the
 * backward pass's kernels read them (0 when that pass reads them in place). */
size_t pf_lowrank_conv_saved_weights_bytes(const pf_conv_desc *d);

/* T = Uk * X (k x k, stride, pad), Y = Vp * T (1x1).  T_save nullable.
 * W_save (nullable, pf_lowrank_conv_saved_weights_bytes(d) bytes): like T_save a
 * tensor kept for the backward pass -- the forward call's weight re-ordering
 * launch fills it, and a backward call that is handed it (with Uk, Vp
 * unchanged in between) skips its own re-ordering launch. */
int pf_lowrank_conv_fwd(const pf_conv_desc *d, const void *X, const void *Uk,
                        const void *Vp, void *Y, void *T_save /* nullable */,
                        void *W_save /* nullable */,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Given dY[N,Cout,Ho,Wo]:  dT = Vp^T dY (1x1),  dVp[o,q] = sum dY T,
 * dX = transposed k x k convolution of dT with Uk,
 * dUk[q,c,i,j] = sum dT[n,q,y,x] Xpad[n,c,y s+i-p,x s+j-p].
 * T_saved nullable (recomputed); W_saved nullable (the forward call's W_save).
 * dX, dUk, dVp each nullable; dUk, dVp float. */
int pf_lowrank_conv_bwd(const pf_conv_desc *d, const void *X, const void *Uk,
                        const void *Vp, const void *dY,
                        const void *T_saved /* nullable */,
                        const void *W_saved /* nullable */, void *dX,
                        void *dUk, void *dVp, int accumulate, void *workspace,
                        size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------ */
/* Layer epilogues: what the paper's models put directly after a        */
/* factorized layer, applied where the layer's output is formed, and    */
/* the matching step of the backward pass.                              */
/*                                                                      */
/* Linear (Section 2.4: FFN(x) = max(0, x W1 + b1) W2 + b2; each        */
/* sub-layer of a Transformer block sits inside a residual connection): */
/*   Z = (X V) U^T + bias + residual,   Y = act(Z)                      */
/*   residual: nullable, [M x out] in dtype.  act: pf_activation.       */
/* Backward takes dZ = dL/dZ where pf_lowrank_linear_bwd takes dY (for  */
/* PF_ACT_NONE they are the same tensor; a residual input receives dZ   */
/* as it is) and forms the gradient the layer BELOW needs:              */
/*   dX = (dZ U V^T + dX_add) * [X > 0]                                 */
/*   dX_add: nullable [M x in] (the gradient arriving over a skip       */
/*   connection that branches off X); the mask only when x_is_relu != 0 */
/*   (X is the output of a ReLU: dX is then dL/dZ of the layer below).  */
/*   dU, dV, dbias as in pf_lowrank_linear_bwd with dY = dZ.            */
/*                                                                      */
/* Convolution (Appendix D: a batch-norm layer after every convolution, */
/* ReLU after it, the shortcut of a ResNet block added before the last  */
/* ReLU), with the statistics fixed (running mean and variance): the    */
/* normalisation is then a per-channel scale and shift,                 */
/*   scale = gamma / sqrt(var + eps), shift = beta - mean * scale:      */
/*   Z[n,o,y,x] = scale[o] (Vp * (Uk * X))[n,o,y,x] + shift[o] + R,     */
/*   Y = act(Z);  scale, shift: float[Cout], each nullable (1 and 0).   */
/* Backward from dZ:  dP = scale dZ, dT = Vp^T dP, dVp = dP T^T,        */
/*   dshift[o] = sum over n,y,x of dZ (float[Cout], nullable),          */
/*   dX = (transposed convolution of dT + dX_add) * [X > 0].            */
/* The scale is a constant here and has no gradient.  A W_saved handed */
/* to the backward call must come from pf_lowrank_conv_fwd_ep called   */
/* with the same scale (the saved copy of the 1x1 filters carries it). */
/*                                                                      */
/* Workspace: the *_fwd_ep calls and pf_lowrank_linear_bwd_ep need what */
/* the plain calls need; pf_lowrank_conv_bwd_ep has its own query.      */
/* Errors as for the plain calls; an unknown act: PF_ERR_UNSUPPORTED.   */
/* ------------------------------------------------------------------ */
typedef enum { PF_ACT_NONE = 0, PF_ACT_RELU = 1 } pf_activation;

int pf_lowrank_linear_fwd_ep(const pf_linear_desc *d, const void *X, const void *V,
                             const void *U, const void *bias /* nullable */,
                             const void *residual /* nullable */, int act,
                             void *Y, void *T_save /* nullable */,
                             void *workspace, size_t workspace_bytes,
                             void *stream);
int pf_lowrank_linear_bwd_ep(const pf_linear_desc *d, const void *X, const void *V,
                             const void *U, const void *dZ,
                             const void *T_saved /* nullable */,
                             const void *dX_add /* nullable */, int x_is_relu,
                             void *dX, void *dU, void *dV, void *dbias,
                             int accumulate, void *workspace,
                             size_t workspace_bytes, void *stream);

size_t pf_lowrank_conv_bwd_ep_workspace_bytes(const pf_conv_desc *d);
int pf_lowrank_conv_fwd_ep(const pf_conv_desc *d, const void *X, const void *Uk,
                           const void *Vp, const void *scale /* nullable */,
                           const void *shift /* nullable */,
                           const void *residual /* nullable */, int act,
                           void *Y, void *T_save /* nullable */,
                           void *W_save /* nullable */, void *workspace,
                           size_t workspace_bytes, void *stream);
int pf_lowrank_conv_bwd_ep(const pf_conv_desc *d, const void *X, const void *Uk,
                           const void *Vp, const void *scale /* nullable */,
                           const void *dZ, const void *T_saved /* nullable */,
                           const void *W_saved /* nullable */,
                           const void *dX_add /* nullable */, int x_is_relu,
                           void *dX, void *dUk, void *dVp,
                           void *dshift /* nullable */, int accumulate,
                           void *workspace, size_t workspace_bytes,
                           void *stream);

/* ------------------------------------------------------------------ */
/* LSTM cell (paper Section 2.3, eq. (2); architecture table of the     */
/* low-rank LSTM in Appendix D).  One time step for a batch of B rows:  */
/*   Tx = x Vx, Th = h_prev Vh,                                        */
/*   z = Tx Ux^T + Th Uh^T + bias   (z[B x 4h], gate blocks i|f|g|o),   */
/*   i,f,o = sigmoid(z), g = tanh(z), c = f c_prev + i g, h = o tanh(c).*/
/*   groups == 4: one factor pair per gate, as eq. (2) has it:          */
/*     Vx[d_in x 4r], gate g reads columns g r..(g+1) r-1 of Tx;        */
/*   groups == 1: the stacked 4h x d_in matrix is one rank-r product:   */
/*     Vx[d_in x r] shared by the gates.                                */
/*   Ux, Uh are [4h x r] in both cases; bias[4h] is the sum of the      */
/*   equation's two bias vectors.  dtype must be PF_F32.                */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t B, d_in, h, r;
    int groups;   /* 1 or 4 */
    int dtype;    /* PF_F32 */
    int has_bias;
} pf_lstm_desc;

size_t pf_lowrank_lstm_cell_fwd_workspace_bytes(const pf_lstm_desc *d);
size_t pf_lowrank_lstm_cell_bwd_workspace_bytes(const pf_lstm_desc *d);

/* Outputs h_out[B x h], c_out[B x h]; saved for backward: gates_save[B x 4h]
 * (activated i|f|g|o), Tx_save, Th_save [B x groups r] -- all three required. */
int pf_lowrank_lstm_cell_fwd(const pf_lstm_desc *d, const void *x,
                             const void *h_prev, const void *c_prev,
                             const void *Vx, const void *Ux, const void *Vh,
                             const void *Uh, const void *bias /* nullable */,
                             void *h_out, void *c_out, void *gates_save,
                             void *Tx_save, void *Th_save, void *workspace,
                             size_t workspace_bytes, void *stream);

/* One step of back-propagation through time.  dh = dL/dh_t (from the layer
 * above plus from step t+1), dc_next = dL/dc_t from step t+1 (NULL = 0).
 * Outputs dx (nullable), dh_prev, dc_prev and the float parameter gradients
 * dVx, dUx, dVh, dUh, dbias (dbias nullable), overwritten or accumulated. */
int pf_lowrank_lstm_cell_bwd(const pf_lstm_desc *d, const void *x,
                             const void *h_prev, const void *c_prev,
                             const void *c_out, const void *gates_saved,
                             const void *Tx_saved, const void *Th_saved,
                             const void *Vx, const void *Ux, const void *Vh,
                             const void *Uh, const void *dh,
                             const void *dc_next /* nullable */,
                             void *dx /* nullable */, void *dh_prev,
                             void *dc_prev, void *dVx, void *dUx, void *dVh,
                             void *dUh, void *dbias /* nullable */,
                             int accumulate, void *workspace,
                             size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------ */
/* Factorized LSTM layer over a whole sequence (Section 2.3, eq. (2)     */
/* applied for t = 0 .. T-1 with h_t, c_t fed to step t+1), fp32.       */
/* Same arithmetic as T calls of the cell; the input path x_t Vx Ux^T   */
/* does not depend on the recurrence and is computed for all time steps */
/* at once, and the parameter gradients are formed once over all steps. */
/*   x[T,B,d_in]; h0, c0 [B,h]; factors and bias as for the cell.       */
/* These run on the small-batch schedule of the stack entry points      */
/* below (a sequence is a stack of one layer) and share its limits:     */
/* B <= 32 and d_in, h, r >= 4, otherwise PF_ERR_UNSUPPORTED -- larger   */
/* batches go step by step through the cell entry points, which take    */
/* any B.                                                               */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t T, B, d_in, h, r;
    int groups;   /* 1 or 4 */
    int dtype;    /* PF_F32 */
    int has_bias;
} pf_lstm_seq_desc;

size_t pf_lowrank_lstm_seq_fwd_workspace_bytes(const pf_lstm_seq_desc *d);
size_t pf_lowrank_lstm_seq_bwd_workspace_bytes(const pf_lstm_seq_desc *d);

/* Outputs h_all, c_all [T,B,h] (h_all[t] = h_t); saved for backward:
 * gates_all[T,B,4h] (activated i|f|g|o), Tx_all, Th_all [T,B,groups r].  All
 * device pointers, all required (bias nullable); T == 0 or B == 0: nothing is
 * done.  Errors as for the cell, plus the limits stated above. */
int pf_lowrank_lstm_seq_fwd(const pf_lstm_seq_desc *d, const void *x,
                            const void *h0, const void *c0, const void *Vx,
                            const void *Ux, const void *Vh, const void *Uh,
                            const void *bias /* nullable */, void *h_all,
                            void *c_all, void *gates_all, void *Tx_all,
                            void *Th_all, void *workspace,
                            size_t workspace_bytes, void *stream);

/* Back-propagation through time.  dh_all[T,B,h] = dL/dh_t arriving from
 * above at every step; dhT, dcT [B,h] = gradients arriving at the final state
 * (NULL = 0).  Outputs dx_all[T,B,d_in] (nullable), dh0, dc0 [B,h] and the
 * float parameter gradients (dbias nullable), overwritten or accumulated. */
int pf_lowrank_lstm_seq_bwd(const pf_lstm_seq_desc *d, const void *x,
                            const void *h0, const void *c0, const void *h_all,
                            const void *c_all, const void *gates_all,
                            const void *Tx_all, const void *Th_all,
                            const void *Vx, const void *Ux, const void *Vh,
                            const void *Uh, const void *dh_all,
                            const void *dhT /* nullable */,
                            const void *dcT /* nullable */,
                            void *dx_all /* nullable */, void *dh0, void *dc0,
                            void *dVx, void *dUx, void *dVh, void *dUh,
                            void *dbias /* nullable */, int accumulate,
                            void *workspace, size_t workspace_bytes,
                            void *stream);

/* ------------------------------------------------------------------ */
/* A stack of `layers` factorized LSTM layers over a sequence (the      */
/* 2-layer language model of Appendix D; eq. (2) per layer, layer l > 0 */
/* reading h_all of layer l - 1).  The result is that of running        */
/* pf_lowrank_lstm_seq_* layer after layer; the steps are scheduled     */
/* along the diagonals l + t = const, which shortens the chain of       */
/* dependent launches from T * layers steps to T + layers - 1.          */
/* Layer 0 has d_in inputs, the others h; every layer has the same h, r */
/* and groups.  fp32, B <= 32, 1 <= layers <= 4, every extent >= 4.     */
/* Per-layer tensors are passed as HOST arrays of `layers` DEVICE       */
/* pointers (the arrays are read during the call only); shapes per      */
/* layer as for the sequence entry points.                              */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t T, B, d_in, h, r;
    int groups;   /* 1 or 4 */
    int layers;   /* 1..4 */
    int dtype;    /* PF_F32 */
    int has_bias;
} pf_lstm_stack_desc;

size_t pf_lowrank_lstm_stack_fwd_workspace_bytes(const pf_lstm_stack_desc *d);
size_t pf_lowrank_lstm_stack_bwd_workspace_bytes(const pf_lstm_stack_desc *d);

/* x[T,B,d_in] device.  h0, c0, Vx, Ux, Vh, Uh, bias (array nullable when
 * has_bias == 0): inputs per layer; h_all, c_all, gates_all, Tx_all, Th_all:
 * outputs per layer (h_all[layers-1] is the output of the stack).  T == 0 or
 * B == 0: nothing is done.  Errors as for the cell. */
int pf_lowrank_lstm_stack_fwd(const pf_lstm_stack_desc *d, const void *x,
                              const void *const *h0, const void *const *c0,
                              const void *const *Vx, const void *const *Ux,
                              const void *const *Vh, const void *const *Uh,
                              const void *const *bias /* nullable */,
                              void *const *h_all, void *const *c_all,
                              void *const *gates_all, void *const *Tx_all,
                              void *const *Th_all, void *workspace,
                              size_t workspace_bytes, void *stream);

/* dh_top[T,B,h] = dL/dh_t of the LAST layer arriving from above at every
 * step; dhT, dcT (arrays and entries nullable = 0): gradients arriving at each
 * layer's final state.  Outputs: dx_all[T,B,d_in] (nullable), dh0, dc0 per
 * layer, and the float parameter gradients per layer (dbias array nullable),
 * overwritten or accumulated. */
int pf_lowrank_lstm_stack_bwd(const pf_lstm_stack_desc *d, const void *x,
                              const void *const *h0, const void *const *c0,
                              const void *const *h_all,
                              const void *const *c_all,
                              const void *const *gates_all,
                              const void *const *Tx_all,
                              const void *const *Th_all,
                              const void *const *Vx, const void *const *Ux,
                              const void *const *Vh, const void *const *Uh,
                              const void *dh_top,
                              const void *const *dhT /* nullable */,
                              const void *const *dcT /* nullable */,
                              void *dx_all /* nullable */, void *const *dh0,
                              void *const *dc0, void *const *dVx,
                              void *const *dUx, void *const *dVh,
                              void *const *dUh,
                              void *const *dbias /* nullable */,
                              int accumulate, void *workspace,
                              size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------ */
/* Truncated-SVD factor initialisation (Algorithm 1, the step before    */
/* the factorized layers are trained): W[m x n] (fp32, row-major) ->    */
/*   U[m x r] = Ut_r S_r^(1/2),  V[n x r] = Vt_r S_r^(1/2)  (fp32),     */
/* so that U V^T is the best rank-r approximation of W; sigma (nullable)*/
/* receives all min(m, n) singular values in descending order.          */
/* One-sided Jacobi in double precision; factors are unique only up to  */
/* the sign of each column pair.  r <= min(m, n) <= 8192 (else          */
/* PF_ERR_SHAPE / PF_ERR_UNSUPPORTED).  For a convolution unroll        */
/* W[c_out, c_in, k, k] to [c_in k^2, c_out] first (Section 2.2).       */
/* Sweeps stop once a whole sweep found every column pair orthogonal to */
/* min(m,n)-independent rounding level (max(m,n) * 2^-52 relative); at  */
/* most 24 sweeps run.  The call is asynchronous, so convergence cannot */
/* come back in the status: info (nullable, DEVICE int[2]) receives     */
/* info[0] = sweeps that ran, info[1] = rotations applied in the last   */
/* of them -- 0 means converged; anything else means the 24 sweeps did  */
/* not suffice and the factors are approximate.                         */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t m, n, r;
} pf_svd_desc;

size_t pf_svd_split_workspace_bytes(const pf_svd_desc *d);
int pf_svd_split(const pf_svd_desc *d, const void *W, void *U, void *V,
                 void *sigma /* nullable */, void *info /* nullable */,
                 void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------ */
/* Dense (un-factorized) comparators, for benchmarks only: the layers   */
/* of Section 2.1 / 2.2 before factorization, on the same tiling code.  */
/*   linear: W[out x in];  conv: Wd[Cout,Cin,k,k].                      */
/* ------------------------------------------------------------------ */
size_t pf_dense_linear_workspace_bytes(const pf_linear_desc *d);
int pf_dense_linear_fwd(const pf_linear_desc *d, const void *X, const void *W,
                        const void *bias, void *Y, void *workspace,
                        size_t workspace_bytes, void *stream);
int pf_dense_linear_bwd(const pf_linear_desc *d, const void *X, const void *W,
                        const void *dY, void *dX, void *dW, void *dbias,
                        int accumulate, void *workspace, size_t workspace_bytes,
                        void *stream);
size_t pf_dense_conv_workspace_bytes(const pf_conv_desc *d);
int pf_dense_conv_fwd(const pf_conv_desc *d, const void *X, const void *Wd,
                      void *Y, void *workspace, size_t workspace_bytes,
                      void *stream);
int pf_dense_conv_bwd(const pf_conv_desc *d, const void *X, const void *Wd,
                      const void *dY, void *dX, void *dWd, int accumulate,
                      void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------ */
/* Per-kernel timing (HIP events recorded around every kernel launch on */
/* the launch stream while enabled).  Not thread-safe; for benchmarks.  */
/* While enabled every launch creates two hipEvents (host objects), so  */
/* do not enable it under stream capture; pf_timing_collect() blocks    */
/* the calling thread until the recorded events have completed.         */
/* ------------------------------------------------------------------ */
void pf_timing_enable(int on);
/* Synchronises the recorded events, adds them to the totals and returns the
 * number of distinct kernels seen so far. */
int pf_timing_collect(void);
/* Entry i of the totals: name (static string), launches, total milliseconds. */
int pf_timing_entry(int i, const char **name, int64_t *launches, double *total_ms);
void pf_timing_reset(void);

#ifdef __cplusplus
}
#endif
#endif /* PUFFERFISH_H */
