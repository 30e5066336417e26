// Layer epilogues: what follows a factorized layer in the paper's models, and its backward.
//   linear (Section 2.4, FFN(x) = max(0, x W1 + b1) W2 + b2, and the residual connection around a sub-layer):
//       Z = T U^T + b + R,  Y = act(Z);      backward from dZ: dX = (dZ U V^T + dX_add) [X > 0]
//   convolution (Appendix D: batch norm after every convolution, ReLU, ResNet shortcut), statistics fixed:
//       Z = scale[o] P + shift[o] + R,  Y = act(Z);   backward from dZ: dP = scale dZ, dshift = sum dZ,
//       dX = (transposed convolution of dT + dX_add) [X > 0]
// The entry points run the layer's own kernels and apply the epilogue element-wise afterwards (one more pass over
// the output); where the layer runs on the fused chain kernels those apply it as they store (pf_conv_chain.hip,
// pf_linear_chain.hip) and nothing is launched here.
#include "pf_epilogue.h"

namespace pf {

template <typename T>
__device__ __forceinline__ void load8(const T *p, float (&f)[8]);
template <>
__device__ __forceinline__ void load8<float>(const float *p, float (&f)[8])
{
    const float4 a = *(const float4 *)p, b = *(const float4 *)(p + 4);
    f[0] = a.x, f[1] = a.y, f[2] = a.z, f[3] = a.w, f[4] = b.x, f[5] = b.y, f[6] = b.z, f[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<bf16_t>(const bf16_t *p, float (&f)[8])
{
    const uint4 v = *(const uint4 *)p;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = bf16_bits_to_float((uint16_t)w[e]);
        f[2 * e + 1] = bf16_bits_to_float((uint16_t)(w[e] >> 16));
    }
}
template <typename T>
__device__ __forceinline__ void store8(T *p, const float (&f)[8]);
template <>
__device__ __forceinline__ void store8<float>(float *p, const float (&f)[8])
{
    *(float4 *)p = make_float4(f[0], f[1], f[2], f[3]);
    *(float4 *)(p + 4) = make_float4(f[4], f[5], f[6], f[7]);
}
template <>
__device__ __forceinline__ void store8<bf16_t>(bf16_t *p, const float (&f)[8])
{
    *(uint4 *)p = make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                             pack_bf16x2(f[6], f[7]));
}

// Y <- act(scale[c] Y + shift[c] + R), channel c of element e = (e / inner) % C.  Eight elements per thread
// (16-byte accesses; every tensor starts 16-byte aligned), the ragged end element by element.
template <typename T>
__global__ __launch_bounds__(256) void ep_fwd_kernel(T *Y, const float *scale, const float *shift, const T *R, int act,
                                                      i64 count, int inner, int C)
{
    const i64 e0 = ((i64)blockIdx.x * 256 + threadIdx.x) * 8;
    if (e0 >= count) return;
    const int n = count - e0 < 8 ? (int)(count - e0) : 8;
    float y[8], r[8];
    if (n == 8) {
        load8<T>(Y + e0, y);
        if (R) load8<T>(R + e0, r);
    } else {
        for (int e = 0; e < n; ++e) {
            y[e] = to_float(Y[e0 + e]);
            if (R) r[e] = to_float(R[e0 + e]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (e < n) {
            float z = y[e];
            if (scale || shift) {
                const int c = (int)(((e0 + e) / inner) % C);
                if (scale) z *= scale[c];
                if (shift) z += shift[c];
            }
            if (R) z += r[e];
            y[e] = act == PF_ACT_RELU ? fmaxf(z, 0.f) : z;
        }
    }
    if (n == 8) {
        store8<T>(Y + e0, y);
    } else {
        for (int e = 0; e < n; ++e) Y[e0 + e] = from_float<T>(y[e]);
    }
}

// dX <- (dX + A) [X > 0]
template <typename T>
__global__ __launch_bounds__(256) void ep_dx_kernel(T *dX, const T *A, const T *X, i64 count)
{
    const i64 e0 = ((i64)blockIdx.x * 256 + threadIdx.x) * 8;
    if (e0 >= count) return;
    const int n = count - e0 < 8 ? (int)(count - e0) : 8;
    float g[8], a[8], x[8];
    if (n == 8) {
        load8<T>(dX + e0, g);
        if (A) load8<T>(A + e0, a);
        if (X) load8<T>(X + e0, x);
    } else {
        for (int e = 0; e < n; ++e) {
            g[e] = to_float(dX[e0 + e]);
            if (A) a[e] = to_float(A[e0 + e]);
            if (X) x[e] = to_float(X[e0 + e]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (e < n) {
            float v = g[e];
            if (A) v += a[e];
            if (X) v = x[e] > 0.f ? v : 0.f;
            g[e] = v;
        }
    }
    if (n == 8) {
        store8<T>(dX + e0, g);
    } else {
        for (int e = 0; e < n; ++e) dX[e0 + e] = from_float<T>(g[e]);
    }
}

// out[o][q] = scale[o] in[o][q]  (the 1x1 filters with the batch-norm scale folded in, for the backward pass)
template <typename T>
__global__ __launch_bounds__(256) void scale_rows_kernel(const T *in, const float *scale, T *out, i64 count, int r)
{
    const i64 i = (i64)blockIdx.x * 256 + threadIdx.x;
    if (i < count) out[i] = from_float<T>(scale[i / r] * to_float(in[i]));
}

// dVp[o][q] (+)= scale[o] raw[o][q]
__global__ __launch_bounds__(256) void dvp_finish_kernel(const float *raw, const float *scale, float *dVp, i64 count, int r,
                                                          int accumulate)
{
    const i64 i = (i64)blockIdx.x * 256 + threadIdx.x;
    if (i < count) {
        const float v = scale[i / r] * raw[i];
        dVp[i] = accumulate ? dVp[i] + v : v;
    }
}

// out[c] (+)= sum over images and pixels of dZ[n][c][p]: one workgroup per channel, fixed summation order.
// Planes that are a whole number of 16-byte pieces are read eight (bf16) or four (float) elements at a time.
template <typename T>
__global__ __launch_bounds__(256) void channel_sum_kernel(const T *dZ, float *out, int N, int C, int HW, int accumulate)
{
    const int c = blockIdx.x, tid = threadIdx.x;
    constexpr int V = 16 / sizeof(T);
    float acc = 0.f;
    if (HW % V == 0) {
        const int pv = HW / V; // pieces per plane
        for (i64 i = tid; i < (i64)N * pv; i += 256) {
            const int n = (int)(i / pv), q = (int)(i - (i64)n * pv);
            const T *src = dZ + ((i64)n * C + c) * HW + (i64)q * V;
            if (sizeof(T) == 2) {
                float f[8];
                load8<T>(src, f);
                acc += ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7]));
            } else {
                const float4 v = *(const float4 *)src;
                acc += (v.x + v.y) + (v.z + v.w);
            }
        }
    } else {
        for (i64 i = tid; i < (i64)N * HW; i += 256) {
            const int n = (int)(i / HW), p = (int)(i - (i64)n * HW);
            acc += to_float(dZ[((i64)n * C + c) * HW + p]);
        }
    }
    __shared__ float red[256];
    red[tid] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) out[c] = accumulate ? out[c] + red[0] : red[0];
}

template <typename T>
int launch_ep_fwd(hipStream_t s, void *Y, const float *scale, const float *shift, const void *R, int act, i64 count,
                  int inner, int C)
{
    int st = PF_OK;
    if (count <= 0 || (!scale && !shift && !R && act == PF_ACT_NONE)) return st;
    PF_LAUNCH(st, "epilogue_fwd", ep_fwd_kernel<T>, dim3((unsigned)((count + 2047) / 2048)), dim3(256), s, (T *)Y, scale,
              shift, (const T *)R, act, count, inner, C);
    return st;
}

template <typename T>
int launch_ep_dx(hipStream_t s, void *dX, const void *A, const void *X, i64 count)
{
    int st = PF_OK;
    if (count <= 0 || !dX || (!A && !X)) return st;
    PF_LAUNCH(st, "epilogue_dx", ep_dx_kernel<T>, dim3((unsigned)((count + 2047) / 2048)), dim3(256), s, (T *)dX,
              (const T *)A, (const T *)X, count);
    return st;
}

int ep_fwd(hipStream_t s, int dtype, void *Y, const float *scale, const float *shift, const void *R, int act, i64 count,
           int inner, int C)
{
    return dtype == PF_F32 ? launch_ep_fwd<float>(s, Y, scale, shift, R, act, count, inner, C)
                           : launch_ep_fwd<bf16_t>(s, Y, scale, shift, R, act, count, inner, C);
}

int ep_dx(hipStream_t s, int dtype, void *dX, const void *A, const void *X, i64 count)
{
    return dtype == PF_F32 ? launch_ep_dx<float>(s, dX, A, X, count) : launch_ep_dx<bf16_t>(s, dX, A, X, count);
}

static bool bad_act(int act) { return act != PF_ACT_NONE && act != PF_ACT_RELU; }

// extra workspace of the convolution's backward epilogue: the scaled 1x1 filters and the unscaled dVp
static size_t conv_ep_extra(const pf_conv_desc *d)
{
    const size_t el = d->dtype == PF_BF16 ? 2 : 4, n = (size_t)d->Cout * (size_t)d->r;
    return align_up(n * el) + align_up(n * 4);
}

} // namespace pf

using namespace pf;

extern "C" {

int pf_lowrank_linear_fwd_ep(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *bias,
                             const void *residual, int act, void *Y, void *T_save, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    if (bad_act(act)) return PF_ERR_UNSUPPORTED;
    if (any_misaligned({residual}, 16)) return PF_ERR_UNSUPPORTED;
    bool fused = false;
    int st = linear_fwd_entry_ep(d, X, V, U, bias, residual, act, Y, T_save, workspace, workspace_bytes, stream, &fused);
    if (st != PF_OK || fused || d->M == 0) return st;
    return ep_fwd((hipStream_t)stream, d->dtype, Y, nullptr, nullptr, residual, act, d->M * d->out, 1, (int)d->out);
}

int pf_lowrank_linear_bwd_ep(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *dZ,
                             const void *T_saved, const void *dX_add, int x_is_relu, void *dX, void *dU, void *dV,
                             void *dbias, int accumulate, void *workspace, size_t workspace_bytes, void *stream)
{
    if (any_misaligned({dX_add}, 16)) return PF_ERR_UNSUPPORTED;
    bool fused = false;
    int st = linear_bwd_entry_ep(d, X, V, U, dZ, T_saved, dX_add, x_is_relu, dX, dU, dV, dbias, accumulate, workspace,
                                 workspace_bytes, stream, &fused);
    if (st != PF_OK || fused || d->M == 0) return st;
    return ep_dx((hipStream_t)stream, d->dtype, dX, dX_add, x_is_relu ? X : nullptr, d->M * d->in);
}

size_t pf_lowrank_conv_bwd_ep_workspace_bytes(const pf_conv_desc *d)
{
    const size_t base = pf_lowrank_conv_bwd_workspace_bytes(d);
    if (!d || d->Cout <= 0 || d->r <= 0) return base;
    return align_up(base) + conv_ep_extra(d);
}

int pf_lowrank_conv_fwd_ep(const pf_conv_desc *d, const void *X, const void *Uk, const void *Vp, const void *scale,
                           const void *shift, const void *residual, int act, void *Y, void *T_save, void *W_save,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (bad_act(act)) return PF_ERR_UNSUPPORTED;
    if (any_misaligned({residual}, 16) || any_misaligned({scale, shift}, 4)) return PF_ERR_UNSUPPORTED;
    bool fused = false;
    int st = conv_fwd_entry_ep(d, X, Uk, Vp, (const float *)scale, (const float *)shift, residual, act, Y, T_save, W_save,
                               workspace, workspace_bytes, stream, &fused);
    if (st != PF_OK || fused || d->N == 0) return st;
    const i64 Ho = (d->H + 2 * (i64)d->pad - d->k) / d->stride + 1, Wo = (d->W + 2 * (i64)d->pad - d->k) / d->stride + 1;
    return ep_fwd((hipStream_t)stream, d->dtype, Y, (const float *)scale, (const float *)shift, residual, act,
                  d->N * d->Cout * Ho * Wo, (int)(Ho * Wo), (int)d->Cout);
}

int pf_lowrank_conv_bwd_ep(const pf_conv_desc *d, const void *X, const void *Uk, const void *Vp, const void *scale,
                           const void *dZ, const void *T_saved, const void *W_saved, const void *dX_add, int x_is_relu,
                           void *dX, void *dUk, void *dVp, void *dshift, int accumulate, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    if (!d) return PF_ERR_NULL;
    if (any_misaligned({dX_add}, 16) || any_misaligned({scale, dshift}, 4)) return PF_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    const size_t base = pf_lowrank_conv_bwd_workspace_bytes(d);
    const void *Vp_used = Vp;
    void *dVp_used = dVp;
    float *raw = nullptr;
    int st = PF_OK;
    // the chain kernels fold the scale into their own weight re-ordering and gradient sum; any other path runs on
    // a scaled copy of the 1x1 filters and finishes dVp afterwards
    const bool in_kernel = scale && conv_bwd_takes_scale(d, dX != nullptr);
    const bool scaled = !in_kernel && scale && Vp && d->Cout > 0 && d->r > 0 && d->N > 0;
    if (scaled) {
        // dT = Vp^T (scale dZ) = (scale Vp)^T dZ: the backward kernels run on a scaled copy of the 1x1 filters,
        // and dVp = scale (dZ T^T) is finished from the unscaled sum.
        const size_t need = align_up(base) + conv_ep_extra(d);
        if (!workspace || workspace_bytes < need) return PF_ERR_WORKSPACE;
        if (any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED;
        const i64 n = d->Cout * d->r;
        const size_t el = d->dtype == PF_BF16 ? 2 : 4;
        char *extra = (char *)workspace + align_up(base);
        void *Vs = extra;
        raw = (float *)(extra + align_up((size_t)n * el));
        if (d->dtype == PF_F32)
            PF_LAUNCH(st, "scale_filters", scale_rows_kernel<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), s,
                      (const float *)Vp, (const float *)scale, (float *)Vs, n, (int)d->r);
        else if (d->dtype == PF_BF16)
            PF_LAUNCH(st, "scale_filters", scale_rows_kernel<bf16_t>, dim3((unsigned)((n + 255) / 256)), dim3(256), s,
                      (const bf16_t *)Vp, (const float *)scale, (bf16_t *)Vs, n, (int)d->r);
        if (st != PF_OK) return st;
        Vp_used = Vs;
        if (dVp) {
            dVp_used = raw;
            // one accumulate flag serves dUk and dVp: when it is set, the unscaled sum starts from zero instead
            if (accumulate) st = launch_zero_f32(s, raw, n);
            if (st != PF_OK) return st;
        }
        W_saved = nullptr; // the forward call's re-ordered copy holds the unscaled filters
    }
    bool fused = false;
    st = conv_bwd_entry_ep(d, X, Uk, Vp_used, in_kernel ? (const float *)scale : nullptr, dZ, T_saved, W_saved, dX_add,
                           x_is_relu, dX, dUk, dVp_used, accumulate, workspace, workspace_bytes, stream, &fused);
    if (st != PF_OK) return st;
    const i64 Ho = (d->H + 2 * (i64)d->pad - d->k) / d->stride + 1, Wo = (d->W + 2 * (i64)d->pad - d->k) / d->stride + 1;
    if (scaled && dVp) {
        const i64 n = d->Cout * d->r;
        PF_LAUNCH(st, "scale_filter_grads", dvp_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), s,
                  (const float *)raw, (const float *)scale, (float *)dVp, n, (int)d->r, accumulate);
        if (st != PF_OK) return st;
    }
    if (dshift) {
        if (d->N == 0) {
            if (!accumulate) st = launch_zero_f32(s, (float *)dshift, d->Cout);
        } else if (d->dtype == PF_F32) {
            PF_LAUNCH(st, "channel_sums", channel_sum_kernel<float>, dim3((unsigned)d->Cout), dim3(256), s,
                      (const float *)dZ, (float *)dshift, (int)d->N, (int)d->Cout, (int)(Ho * Wo), accumulate);
        } else {
            PF_LAUNCH(st, "channel_sums", channel_sum_kernel<bf16_t>, dim3((unsigned)d->Cout), dim3(256), s,
                      (const bf16_t *)dZ, (float *)dshift, (int)d->N, (int)d->Cout, (int)(Ho * Wo), accumulate);
        }
        if (st != PF_OK) return st;
    }
    if (fused || d->N == 0) return st;
    return ep_dx(s, d->dtype, dX, dX_add, x_is_relu ? X : nullptr, d->N * d->Cin * d->H * d->W);
}

} // extern "C"
