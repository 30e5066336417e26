// Factorized fully connected layer (paper Section 2.1): Y = (X V) U^T + bias and its
// gradients, plus the dense comparator.  Host-side validation, workspace planning and
// dispatch; the any-shape path composes the guarded tile GEMM.
#include "pf_gemm.h"

namespace pf {

// dst[s][col] = sum over the s-th row chunk of src[row * ld + col]
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T *src, float *partial, int rows, int cols, i64 ld,
                                                              int rows_per_chunk)
{
    __shared__ float red[4][64];
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int q = threadIdx.x >> 6;
    const int rbeg = blockIdx.y * rows_per_chunk;
    const int rend = min(rows, rbeg + rows_per_chunk);
    float acc = 0.f;
    if (c < cols)
        for (int r = rbeg + q; r < rend; r += 4) acc += to_float(src[(i64)r * ld + c]);
    red[q][threadIdx.x & 63] = acc;
    __syncthreads();
    if (q == 0 && c < cols)
        partial[(i64)blockIdx.y * cols + c] = red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] +
                                              red[3][threadIdx.x];
}

int colsum_chunks(i64 rows)
{
    i64 c = (rows + 511) / 512;
    return (int)(c > 64 ? 64 : c < 1 ? 1 : c);
}

// out[cols] (+)= column sums of src[rows x cols]; partial holds colsum_chunks(rows) * cols floats.
template <typename T>
int launch_colsum(hipStream_t stream, const T *src, float *partial, float *out, i64 rows, i64 cols, i64 ld,
                  int accumulate)
{
    int status = PF_OK;
    const int chunks = colsum_chunks(rows);
    const int per = (int)((rows + chunks - 1) / chunks);
    dim3 grid((unsigned)((cols + 63) / 64), chunks);
    PF_LAUNCH(status, "colsum_partial", (colsum_partial_kernel<T>), grid, dim3(256), stream, src, partial, (int)rows,
              (int)cols, ld, per);
    if (status != PF_OK) return status;
    return launch_splitk_reduce(stream, partial, out, cols, chunks, accumulate);
}

template int launch_colsum<float>(hipStream_t, const float *, float *, float *, i64, i64, i64, int);
template int launch_colsum<bf16_t>(hipStream_t, const bf16_t *, float *, float *, i64, i64, i64, int);

// ------------------------------------------------------------ validation
static int check_linear_desc(const pf_linear_desc *d)
{
    if (!d) return PF_ERR_NULL;
    if (d->dtype != PF_F32 && d->dtype != PF_BF16) return PF_ERR_UNSUPPORTED;
    if (d->M < 0 || d->in <= 0 || d->out <= 0 || d->r <= 0) return PF_ERR_SHAPE;
    const i64 lim = 0x7fffffffLL;
    if (d->M > lim || d->in > lim || d->out > lim || d->r > lim) return PF_ERR_SHAPE;
    if (d->M * d->in > (lim << 4) || d->M * d->out > (lim << 4)) return PF_ERR_SHAPE;
    return PF_OK;
}

// ---------------------------------------------------------- workspace plan
struct LinearPlan {
    int ks_dU, ks_dV;
    size_t fwd_bytes, bwd_bytes;
    size_t n_T, n_dT, n_part;
};

static LinearPlan plan_linear(const pf_linear_desc *d)
{
    LinearPlan p;
    p.ks_dU = choose_ksplit(d->out, d->r, d->M);
    p.ks_dV = choose_ksplit(d->in, d->r, d->M);
    p.n_T = (size_t)(d->M * d->r);
    p.n_dT = p.n_T;
    size_t part_dU = (size_t)p.ks_dU * d->out * d->r, part_dV = (size_t)p.ks_dV * d->in * d->r;
    size_t part_db = (size_t)colsum_chunks(d->M) * d->out;
    p.n_part = part_dU > part_dV ? part_dU : part_dV;
    if (part_db > p.n_part) p.n_part = part_db;
    p.fwd_bytes = align_up(p.n_T * sizeof(float));
    p.bwd_bytes = align_up(p.n_T * sizeof(float)) + align_up(p.n_dT * sizeof(float)) + align_up(p.n_part * sizeof(float));
    return p;
}

// ------------------------------------------------------------- any-shape
template <typename T>
static int linear_fwd_generic(const pf_linear_desc *d, const T *X, const T *V, const T *U, const T *bias, T *Y,
                              T *T_save, Workspace &ws, hipStream_t s)
{
    const int M = (int)d->M, in = (int)d->in, out = (int)d->out, r = (int)d->r;
    float *Tws = ws.take<float>((size_t)M * r);
    int st = launch_gemm_generic<T, true, false>(
        "linear_T=X*V", s, GemmShape{M, r, in, 1, 1}, OpA_RowMajor<T>{X, in, 0}, OpB_KN<T>{V, r, 0, 0},
        EpiRowMajor<float, T>{Tws, T_save, r, nullptr, 0});
    if (st != PF_OK) return st;
    return launch_gemm_generic<T, true, true>(
        "linear_Y=T*Ut", s, GemmShape{M, out, r, 1, 1}, OpA_RowMajor<float>{Tws, r, 0}, OpB_NK<T>{U, r, 0},
        EpiRowMajor<T, T>{Y, nullptr, out, d->has_bias ? bias : nullptr, 0});
}

template <typename T>
static int linear_bwd_generic(const pf_linear_desc *d, const T *X, const T *V, const T *U, const T *dY,
                              const T *T_saved, T *dX, float *dU, float *dV, float *dbias, int accumulate,
                              Workspace &ws, hipStream_t s)
{
    const int M = (int)d->M, in = (int)d->in, out = (int)d->out, r = (int)d->r;
    const LinearPlan p = plan_linear(d);
    float *Tws = ws.take<float>(p.n_T);
    float *dTws = ws.take<float>(p.n_dT);
    float *part = ws.take<float>(p.n_part);
    int st = PF_OK;
    if (M == 0) {
        if (!accumulate) {
            st = launch_zero_f32(s, dU, (i64)out * r);
            if (st == PF_OK) st = launch_zero_f32(s, dV, (i64)in * r);
            if (st == PF_OK && d->has_bias) st = launch_zero_f32(s, dbias, out);
        }
        return st;
    }
    if (dU && !T_saved) {
        st = launch_gemm_generic<T, true, false>(
            "linear_T=X*V", s, GemmShape{M, r, in, 1, 1}, OpA_RowMajor<T>{X, in, 0}, OpB_KN<T>{V, r, 0, 0},
            EpiRowMajor<float, float>{Tws, nullptr, r, nullptr, 0});
        if (st != PF_OK) return st;
    }
    if (dX || dV) {
        st = launch_gemm_generic<T, true, false>(
            "linear_dT=dY*U", s, GemmShape{M, r, out, 1, 1}, OpA_RowMajor<T>{dY, out, 0}, OpB_KN<T>{U, r, 0, 0},
            EpiRowMajor<float, float>{dTws, nullptr, r, nullptr, 0});
        if (st != PF_OK) return st;
    }
    if (dX) {
        st = launch_gemm_generic<T, true, true>(
            "linear_dX=dT*Vt", s, GemmShape{M, in, r, 1, 1}, OpA_RowMajor<float>{dTws, r, 0}, OpB_NK<T>{V, r, 0},
            EpiRowMajor<T, T>{dX, nullptr, in, nullptr, 0});
        if (st != PF_OK) return st;
    }
    if (dU) {
        const GemmShape g{out, r, M, 1, p.ks_dU};
        const EpiPartial epi{part, r, (i64)out * r};
        if (T_saved)
            st = launch_gemm_generic<T, false, false>("linear_dU=dYt*T", s, g, OpA_ColMajor<T>{dY, out, 0},
                                                      OpB_KN<T>{T_saved, r, 0, 0}, epi);
        else
            st = launch_gemm_generic<T, false, false>("linear_dU=dYt*T", s, g, OpA_ColMajor<T>{dY, out, 0},
                                                      OpB_KN<float>{Tws, r, 0, 0}, epi);
        if (st == PF_OK) st = launch_splitk_reduce(s, part, dU, (i64)out * r, p.ks_dU, accumulate);
        if (st != PF_OK) return st;
    }
    if (dV) {
        st = launch_gemm_generic<T, false, false>("linear_dV=Xt*dT", s, GemmShape{in, r, M, 1, p.ks_dV},
                                                  OpA_ColMajor<T>{X, in, 0}, OpB_KN<float>{dTws, r, 0, 0},
                                                  EpiPartial{part, r, (i64)in * r});
        if (st == PF_OK) st = launch_splitk_reduce(s, part, dV, (i64)in * r, p.ks_dV, accumulate);
        if (st != PF_OK) return st;
    }
    if (d->has_bias && dbias) st = launch_colsum<T>(s, dY, part, dbias, M, out, out, accumulate);
    return st;
}

// ------------------------------------------------------------------ dense
struct DensePlan {
    int ks;
    size_t n_part, bytes;
};
static DensePlan plan_dense_linear(const pf_linear_desc *d)
{
    DensePlan p;
    p.ks = choose_ksplit(d->out, d->in, d->M);
    size_t a = (size_t)p.ks * d->out * d->in, b = (size_t)colsum_chunks(d->M) * d->out;
    p.n_part = a > b ? a : b;
    p.bytes = align_up(p.n_part * sizeof(float));
    return p;
}

template <typename T>
static int dense_linear_fwd_t(const pf_linear_desc *d, const T *X, const T *W, const T *bias, T *Y, hipStream_t s)
{
    const int M = (int)d->M, in = (int)d->in, out = (int)d->out;
    return launch_gemm_generic<T, true, true>("dense_linear_Y=X*Wt", s, GemmShape{M, out, in, 1, 1},
                                              OpA_RowMajor<T>{X, in, 0}, OpB_NK<T>{W, in, 0},
                                              EpiRowMajor<T, T>{Y, nullptr, out, d->has_bias ? bias : nullptr, 0});
}

template <typename T>
static int dense_linear_bwd_t(const pf_linear_desc *d, const T *X, const T *W, const T *dY, T *dX, float *dW,
                              float *dbias, int accumulate, Workspace &ws, hipStream_t s)
{
    const int M = (int)d->M, in = (int)d->in, out = (int)d->out;
    const DensePlan p = plan_dense_linear(d);
    float *part = ws.take<float>(p.n_part);
    int st = PF_OK;
    if (M == 0) {
        if (!accumulate) {
            st = launch_zero_f32(s, dW, (i64)out * in);
            if (st == PF_OK && d->has_bias) st = launch_zero_f32(s, dbias, out);
        }
        return st;
    }
    if (dX) {
        st = launch_gemm_generic<T, true, false>("dense_linear_dX=dY*W", s, GemmShape{M, in, out, 1, 1},
                                                 OpA_RowMajor<T>{dY, out, 0}, OpB_KN<T>{W, in, 0, 0},
                                                 EpiRowMajor<T, T>{dX, nullptr, in, nullptr, 0});
        if (st != PF_OK) return st;
    }
    if (dW) {
        st = launch_gemm_generic<T, false, false>("dense_linear_dW=dYt*X", s, GemmShape{out, in, M, 1, p.ks},
                                                  OpA_ColMajor<T>{dY, out, 0}, OpB_KN<T>{X, in, 0, 0},
                                                  EpiPartial{part, in, (i64)out * in});
        if (st == PF_OK) st = launch_splitk_reduce(s, part, dW, (i64)out * in, p.ks, accumulate);
        if (st != PF_OK) return st;
    }
    if (d->has_bias && dbias) st = launch_colsum<T>(s, dY, part, dbias, M, out, out, accumulate);
    return st;
}

} // namespace pf

using namespace pf;

extern "C" {

size_t pf_lowrank_linear_fwd_workspace_bytes(const pf_linear_desc *d)
{
    if (check_linear_desc(d) != PF_OK) return 0;
    return plan_linear(d).fwd_bytes;
}

size_t pf_lowrank_linear_bwd_workspace_bytes(const pf_linear_desc *d)
{
    if (check_linear_desc(d) != PF_OK) return 0;
    return plan_linear(d).bwd_bytes;
}

int pf_lowrank_linear_fwd(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *bias,
                          void *Y, void *T_save, void *workspace, size_t workspace_bytes, void *stream)
{
    int st = check_linear_desc(d);
    if (st != PF_OK) return st;
    if (!V || !U || (d->has_bias && !bias)) return PF_ERR_NULL;
    if (d->M > 0 && (!X || !Y)) return PF_ERR_NULL;
    const size_t need = plan_linear(d).fwd_bytes;
    if (need > 0 && (!workspace || workspace_bytes < need)) return PF_ERR_WORKSPACE;
    if (d->M == 0) return PF_OK;
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32)
        return linear_fwd_generic<float>(d, (const float *)X, (const float *)V, (const float *)U, (const float *)bias,
                                         (float *)Y, (float *)T_save, ws, s);
    return linear_fwd_generic<bf16_t>(d, (const bf16_t *)X, (const bf16_t *)V, (const bf16_t *)U,
                                      (const bf16_t *)bias, (bf16_t *)Y, (bf16_t *)T_save, ws, s);
}

int pf_lowrank_linear_bwd(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *dY,
                          const void *T_saved, void *dX, void *dU, void *dV, void *dbias, int accumulate,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    int st = check_linear_desc(d);
    if (st != PF_OK) return st;
    if (!V || !U) return PF_ERR_NULL;
    if (d->M > 0 && (!X || !dY)) return PF_ERR_NULL;
    const size_t need = plan_linear(d).bwd_bytes;
    if (need > 0 && (!workspace || workspace_bytes < need)) return PF_ERR_WORKSPACE;
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32)
        return linear_bwd_generic<float>(d, (const float *)X, (const float *)V, (const float *)U, (const float *)dY,
                                         (const float *)T_saved, (float *)dX, (float *)dU, (float *)dV,
                                         (float *)dbias, accumulate, ws, s);
    return linear_bwd_generic<bf16_t>(d, (const bf16_t *)X, (const bf16_t *)V, (const bf16_t *)U,
                                      (const bf16_t *)dY, (const bf16_t *)T_saved, (bf16_t *)dX, (float *)dU,
                                      (float *)dV, (float *)dbias, accumulate, ws, s);
}

size_t pf_dense_linear_workspace_bytes(const pf_linear_desc *d)
{
    if (check_linear_desc(d) != PF_OK) return 0;
    return plan_dense_linear(d).bytes;
}

int pf_dense_linear_fwd(const pf_linear_desc *d, const void *X, const void *W, const void *bias, void *Y,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    (void)workspace;
    (void)workspace_bytes;
    int st = check_linear_desc(d);
    if (st != PF_OK) return st;
    if (!W || (d->has_bias && !bias)) return PF_ERR_NULL;
    if (d->M == 0) return PF_OK;
    if (!X || !Y) return PF_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32)
        return dense_linear_fwd_t<float>(d, (const float *)X, (const float *)W, (const float *)bias, (float *)Y, s);
    return dense_linear_fwd_t<bf16_t>(d, (const bf16_t *)X, (const bf16_t *)W, (const bf16_t *)bias, (bf16_t *)Y, s);
}

int pf_dense_linear_bwd(const pf_linear_desc *d, const void *X, const void *W, const void *dY, void *dX, void *dW,
                        void *dbias, int accumulate, void *workspace, size_t workspace_bytes, void *stream)
{
    int st = check_linear_desc(d);
    if (st != PF_OK) return st;
    if (!W) return PF_ERR_NULL;
    if (d->M > 0 && (!X || !dY)) return PF_ERR_NULL;
    const size_t need = plan_dense_linear(d).bytes;
    if (!workspace || workspace_bytes < need) return PF_ERR_WORKSPACE;
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32)
        return dense_linear_bwd_t<float>(d, (const float *)X, (const float *)W, (const float *)dY, (float *)dX,
                                         (float *)dW, (float *)dbias, accumulate, ws, s);
    return dense_linear_bwd_t<bf16_t>(d, (const bf16_t *)X, (const bf16_t *)W, (const bf16_t *)dY, (bf16_t *)dX,
                                      (float *)dW, (float *)dbias, accumulate, ws, s);
}

} // extern "C"
