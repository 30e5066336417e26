// Layer epilogues (bias / fixed-statistics batch norm, residual input, ReLU and their backward): the element-wise
// kernels, and the layer entry points that take an epilogue and report whether their kernels applied it.
#pragma once
#include "pf_gemm.h"

namespace pf {

// Y <- act(scale[c] Y + shift[c] + R) in place; channel of element e = (e / inner) % C.  Nothing to do: no launch.
int ep_fwd(hipStream_t s, int dtype, void *Y, const float *scale, const float *shift, const void *R, int act, i64 count,
           int inner, int C);
// dX <- (dX + A) [X > 0] in place (A, X nullable).
int ep_dx(hipStream_t s, int dtype, void *dX, const void *A, const void *X, i64 count);

// The layers' entry points with an epilogue.  *fused is set when the layer's own kernels applied the epilogue as
// they stored (then the caller launches nothing more), and left false when the plain result was written.
int linear_fwd_entry_ep(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *bias,
                        const void *residual, int act, void *Y, void *T_save, void *workspace, size_t workspace_bytes,
                        void *stream, bool *fused);
int linear_bwd_entry_ep(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *dZ,
                        const void *T_saved, const void *dX_add, int x_is_relu, void *dX, void *dU, void *dV,
                        void *dbias, int accumulate, void *workspace, size_t workspace_bytes, void *stream, bool *fused);
int conv_fwd_entry_ep(const pf_conv_desc *d, const void *X, const void *Uk, const void *Vp, const float *scale,
                      const float *shift, const void *residual, int act, void *Y, void *T_save, void *W_save,
                      void *workspace, size_t workspace_bytes, void *stream, bool *fused);
// scale: honoured only when conv_bwd_takes_scale(d, dX != NULL); otherwise pass NULL and scale beforehand.
int conv_bwd_entry_ep(const pf_conv_desc *d, const void *X, const void *Uk, const void *Vp, const float *scale,
                      const void *dZ, const void *T_saved, const void *W_saved, const void *dX_add, int x_is_relu,
                      void *dX, void *dUk, void *dVp, int accumulate, void *workspace, size_t workspace_bytes,
                      void *stream, bool *fused);
bool conv_bwd_takes_scale(const pf_conv_desc *d, bool want_dX);

} // namespace pf
