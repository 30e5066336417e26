// Factorized fully connected layer (paper Section 2.1): Y = (X V) U^T + bias and its
// gradients, plus the dense comparator.  Host-side validation, workspace planning and
// dispatch; the any-shape path composes the guarded tile GEMM.
#include "pf_conv_chain.h"
#include "pf_linear_chain.h"
#include "pf_skinny.h"
#include "pf_linear_small.h"
#include "pf_conv_wgrad.h"
#include <mutex>
#include "pf_gemm.h"
#include "pf_epilogue.h"

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

// bf16, cols a multiple of 8: a thread owns 8 neighbouring columns (one 16-byte load per row) and every 32nd
// row of the chunk; the 32 row-lanes of a column group are added through LDS in a fixed order.
__global__ __launch_bounds__(256) void colsum_partial_bf16x8_kernel(const uint16_t *src, float *partial, int rows, int cols,
                                                                     i64 ld, int rows_per_chunk)
{
    __shared__ float red[32][64 + 1];
    const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3; // column group within the block's 64 columns, row lane
    const int c0 = blockIdx.x * 64 + 8 * cg;
    const int rbeg = blockIdx.y * rows_per_chunk, rend = min(rows, rbeg + rows_per_chunk);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (c0 < cols) {
#pragma unroll 4
        for (int r = rbeg + rl; r < rend; r += 32) {
            const uint4 v = *(const uint4 *)(src + (i64)r * ld + c0);
            const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[2 * e] += __uint_as_float(d[e] << 16);
                acc[2 * e + 1] += __uint_as_float(d[e] & 0xffff0000u);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[rl][8 * cg + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < 64 && blockIdx.x * 64 + threadIdx.x < cols) {
        float sum = 0.f;
#pragma unroll
        for (int q = 0; q < 32; ++q) sum += red[q][threadIdx.x];
        partial[(i64)blockIdx.y * cols + blockIdx.x * 64 + threadIdx.x] = sum;
    }
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
    if (sizeof(T) == 2 && cols % 8 == 0 && ld % 8 == 0) {
        PF_LAUNCH(status, "colsum_partial", colsum_partial_bf16x8_kernel, grid, dim3(256), stream,
                  (const uint16_t *)src, partial, (int)rows, (int)cols, ld, per);
    } else {
        PF_LAUNCH(status, "colsum_partial", (colsum_partial_kernel<T>), grid, dim3(256), stream, src, partial,
                  (int)rows, (int)cols, ld, per);
    }
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
    if (d->wgrad_dtype != PF_F32) return PF_ERR_UNSUPPORTED; // parameter gradients are float sums
    if (d->M < 0 || d->in <= 0 || d->out <= 0 || d->r <= 0) return PF_ERR_SHAPE;
    const i64 lim = 0x7fffffffLL;
    if (d->M > lim || d->in > lim || d->out > lim || d->r > lim) return PF_ERR_SHAPE;
    if (d->M * d->in > (lim << 4) || d->M * d->out > (lim << 4)) return PF_ERR_SHAPE;
    return PF_OK;
}

// What the 32-row chain kernel applies as its output leaves (all optional; *used reports that it did).
struct LinEpilogue {
    const void *add, *mask;
    int relu;
    bool *used;
};

int linear_fwd_entry(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *bias, void *Y,
                     void *T_save, void *workspace, size_t workspace_bytes, void *stream, int align,
                     const LinEpilogue *ep = nullptr);
int linear_bwd_entry(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *dY,
                     const void *T_saved, void *dX, void *dU, void *dV, void *dbias, int accumulate, void *workspace,
                     size_t workspace_bytes, void *stream, int align, const LinEpilogue *ep = nullptr);

// ---------------------------------------------------------- workspace plan
struct LinearPlan {
    int ks_dU, ks_dV;
    size_t fwd_bytes, bwd_bytes;
    size_t n_T, n_dT, n_part;
    bool fused;         // bf16 and shapes the fused chain / factor-gradient kernels take
    bool chain2;        // ... and the rank the 32-row chain kernel is built for: no weight re-ordering pass
    size_t n_colsum;    // per-tile column sums of dY (bias gradient), floats
    int wg_groups, wg_ipg; // row-tile groups of the factor-gradient kernel and tiles per group
    int wg_cols;           // columns per workgroup of that kernel
    bool skinny;           // fp32 with at most 128 rows: the weight-streaming kernels of the LSTM cell
    size_t n_part_sk;      // their slice sums, floats
    bool small;            // fp32 with at most 128 rows and dimensions in whole tiles: two launches per direction
    size_t n_small;        // slices of the rank-r intermediate(s) between them, floats
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
    p.fused = d->dtype == PF_BF16 && linear_chain_supported(d->in, d->out, d->r);
    p.skinny = d->dtype == PF_F32 && d->M > 0 && d->M <= 4 * SK_MAX_ROWS && d->in >= 4 && d->out >= 4 &&
               d->r >= 4;
    p.n_part_sk = 0;
    if (p.skinny) {
        SkinnyArgs a;
        const int M = (int)d->M, in = (int)d->in, out = (int)d->out, r = (int)d->r;
        const size_t n1 = skinny_rows(M, nullptr, in, nullptr, r, in, r, nullptr, a);   // T = X V
        const size_t n2 = skinny_rows(M, nullptr, r, nullptr, r, r, out, nullptr, a);   // Y = T U^T
        const size_t n3 = skinny_rows(M, nullptr, out, nullptr, r, out, r, nullptr, a); // dT = dY U
        const size_t n4 = skinny_rows(M, nullptr, r, nullptr, r, r, in, nullptr, a);    // dX = dT V^T
        const size_t f = n1 > n2 ? n1 : n2, b = n3 > n4 ? n3 : n4;
        p.n_part_sk = f > b ? f : b;
        const size_t fwd = align_up(p.n_T * sizeof(float)) + align_up(p.n_part_sk * sizeof(float));
        const size_t bwd = 2 * align_up(p.n_T * sizeof(float)) + align_up(p.n_part_sk * sizeof(float));
        if (fwd > p.fwd_bytes) p.fwd_bytes = fwd;
        if (bwd > p.bwd_bytes) p.bwd_bytes = bwd;
    }
    p.small = d->dtype == PF_F32 && linear_small_supported(d->M, d->in, d->out, d->r);
    p.n_small = p.small ? (size_t)(8 * d->M * d->r) : 0; // at most eight slices per intermediate
    if (p.small) {
        const size_t one = align_up(p.n_small * sizeof(float));
        if (one > p.fwd_bytes) p.fwd_bytes = one;
        if (2 * one > p.bwd_bytes) p.bwd_bytes = 2 * one;
    }
    p.chain2 = p.fused && linear_chain2_supported(d->in, d->out, d->r);
    p.n_colsum = p.chain2 ? (size_t)(2 * ((d->M + LC_ROWS - 1) / LC_ROWS)) * d->out : 0;
    p.wg_groups = p.wg_ipg = 1;
    p.wg_cols = 256;
    if (p.fused) {
        const i64 tiles = (d->M + 63) / 64;
        i64 chunks = d->in / 256 + d->out / 256;
        // workgroups over half the chip, each keeping two 64-row tiles in flight: every group costs a partial sum to
        // write and to add (measured on the Transformer shapes: 0.322 ms per block against 0.328 with 256 and 0.352
        // with 64 here)
        i64 want = 128 / chunks;
        want = want < 1 ? 1 : want > 32 ? 32 : want; // (the cap bounds the partial sums the groups write)
        if (want > tiles) want = tiles > 0 ? tiles : 1;
        p.wg_cols = 256;
        if (chunks * want < 200) { // too few workgroups for the chip: narrower column tiles
            p.wg_cols = 128;
            chunks *= 2;
        }
        p.wg_ipg = (int)((tiles + want - 1) / want);
        if (p.wg_ipg < 1) p.wg_ipg = 1;
        p.wg_groups = (int)((tiles + p.wg_ipg - 1) / p.wg_ipg);
        if (p.wg_groups < 1) p.wg_groups = 1;
        const size_t wmax = (size_t)(d->in > d->out ? d->in : d->out) * d->r;
        const size_t fwd = align_up(wmax * 2);
        const size_t grads = (size_t)p.wg_groups * d->r * (d->in + d->out);
        const size_t part = grads > p.n_part ? grads : p.n_part;
        const size_t bwd = align_up(wmax * 2) + 2 * align_up(p.n_T * 2) + align_up(part * sizeof(float)) +
                           align_up(p.n_colsum * sizeof(float));
        if (fwd > p.fwd_bytes) p.fwd_bytes = fwd;
        if (bwd > p.bwd_bytes) p.bwd_bytes = bwd;
    }
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

// ------------------------------------------------------------- fused (bf16)
// Y = (X V) U^T + bias on the two-stage chain kernel: stage 1 weights = V^T re-ordered into MFMA fragments,
// stage 2 weights = U[out][r] read in place.
static int linear_fwd_fused(const pf_linear_desc *d, const bf16_t *X, const bf16_t *V, const bf16_t *U,
                            const bf16_t *bias, bf16_t *Y, bf16_t *T_save, Workspace &ws, hipStream_t s,
                            const LinEpilogue &ep = LinEpilogue{})
{
    const int in = (int)d->in, out = (int)d->out, r = (int)d->r;
    if (linear_chain2_supported(in, out, r)) {
        LinChainArgs c{(const uint16_t *)X, (const uint16_t *)V, (const uint16_t *)U,
                       d->has_bias ? (const uint16_t *)bias : nullptr, (uint16_t *)Y, (uint16_t *)T_save, nullptr,
                       d->M, in, out};
        c.ep_add = (const uint16_t *)ep.add;
        c.ep_relu = ep.relu;
        if (ep.used) *ep.used = true;
        return launch_linear_chain2(s, "linear_fwd_fused", c);
    }
    uint16_t *w1 = ws.take<uint16_t>((size_t)(in > out ? in : out) * r);
    int st = launch_pack_chain(s, make_pack_w1((const uint16_t *)V, (uint4 *)w1, in, r, 1, 1, r, 0),
                               make_pack_w2(nullptr, nullptr, out, r, 1, 0, 0, 0, 0));
    if (st != PF_OK) return st;
    ChainArgs a{(const uint16_t *)X, (const uint4 *)w1, nullptr, (const uint16_t *)U, (uint16_t *)Y,
                (uint16_t *)T_save,  in,                out,     8,                   8,
                d->M,                d->has_bias ? bias : nullptr};
    return launch_linear_chain(s, "linear_fwd_fused", a, r);
}

// Both factor gradients in one launch, their group sums, and the bias gradient (from the column sums the chain
// kernel left, two rows per 32-row tile, or from dY).
static int linear_wgrads_fused(const pf_linear_desc *d, const LinearPlan &p, const bf16_t *X, const bf16_t *dY,
                               const bf16_t *Tt, const bf16_t *dT16, float *dU, float *dV, float *dbias,
                               const float *colsum, int accumulate, float *part, hipStream_t s)
{
    const int M = (int)d->M, in = (int)d->in, out = (int)d->out, r = (int)d->r;
    const bool want_db = d->has_bias && dbias;
    const int tiles = (M + 63) / 64;
    float *part_dU = part, *part_dV = part + (size_t)p.wg_groups * r * out;
    WgradArgs a1{(const uint16_t *)Tt, (const uint16_t *)dY, dU ? part_dU : nullptr, r, out, 8, 8, tiles, p.wg_ipg,
                 p.wg_groups,          d->M};
    WgradArgs a2{(const uint16_t *)dT16, (const uint16_t *)X, dV ? part_dV : nullptr, r, in, 8, 8, tiles, p.wg_ipg,
                 p.wg_groups,            d->M};
    int st = launch_linear_wgrad_pair(s, a1, a2, p.wg_cols);
    if (st != PF_OK) return st;
    WgradReduceArgs r0{part_dU, dU, p.wg_groups, 1, r, out, 1, r, 0, accumulate};
    WgradReduceArgs r1{part_dV, dV, p.wg_groups, 1, r, in, 1, r, 0, accumulate};
    const ColsumTilesArgs cs{colsum, dbias, 2 * ((M + LC_ROWS - 1) / LC_ROWS), out, accumulate};
    st = launch_wgrad_reduce(s, r0, r1, want_db && colsum ? &cs : nullptr);
    if (st != PF_OK) return st;
    if (want_db && !colsum) st = launch_colsum<bf16_t>(s, dY, part, dbias, M, out, out, accumulate);
    return st;
}

// dT = dY U, dX = dT V^T on the same kernel (stage 1 weights = U^T re-ordered, stage 2 weights = V[in][r] in
// place); then both factor gradients in one launch, their group sums, and the bias gradient.
static int linear_bwd_fused(const pf_linear_desc *d, const LinearPlan &p, const bf16_t *X, const bf16_t *V,
                            const bf16_t *U, const bf16_t *dY, const bf16_t *T_saved, bf16_t *dX, float *dU, float *dV,
                            float *dbias, int accumulate, Workspace &ws, hipStream_t s,
                            const LinEpilogue &ep = LinEpilogue{})
{
    const int M = (int)d->M, in = (int)d->in, out = (int)d->out, r = (int)d->r;
    uint16_t *w1 = ws.take<uint16_t>((size_t)(in > out ? in : out) * r);
    bf16_t *dT16 = ws.take<bf16_t>(p.n_T);
    bf16_t *T16 = ws.take<bf16_t>(p.n_T);
    const size_t grads = (size_t)p.wg_groups * r * (in + out);
    float *part = ws.take<float>(grads > p.n_part ? grads : p.n_part);
    float *colsum = p.chain2 ? ws.take<float>(p.n_colsum) : nullptr;
    const bool want_db = d->has_bias && dbias;
    int st = PF_OK;
    if (dU && !T_saved) { // T was not saved: recompute it
        st = launch_gemm_generic<bf16_t, true, false>(
            "linear_T=X*V", s, GemmShape{M, r, in, 1, 1}, OpA_RowMajor<bf16_t>{X, in, 0}, OpB_KN<bf16_t>{V, r, 0, 0},
            EpiRowMajor<bf16_t, bf16_t>{T16, nullptr, r, nullptr, 0});
        if (st != PF_OK) return st;
    }
    if (p.chain2) {
        LinChainArgs c{(const uint16_t *)dY, (const uint16_t *)U, (const uint16_t *)V, nullptr, (uint16_t *)dX,
                       (uint16_t *)dT16, want_db ? colsum : nullptr, d->M, out, in};
        c.ep_add = (const uint16_t *)ep.add;
        c.ep_mask = (const uint16_t *)ep.mask;
        if (ep.used) *ep.used = true;
        st = launch_linear_chain2(s, "linear_bwd_data_fused", c);
    } else {
        st = launch_pack_chain(s, make_pack_w1((const uint16_t *)U, (uint4 *)w1, out, r, 1, 1, r, 0),
                               make_pack_w2(nullptr, nullptr, in, r, 1, 0, 0, 0, 0));
        if (st != PF_OK) return st;
        ChainArgs a{(const uint16_t *)dY, (const uint4 *)w1, nullptr, (const uint16_t *)V, (uint16_t *)dX,
                    (uint16_t *)dT16,     out,               in,      8,                   8,
                    d->M,                 nullptr};
        st = launch_linear_chain(s, "linear_bwd_data_fused", a, r);
    }
    if (st != PF_OK) return st;
    return linear_wgrads_fused(d, p, X, dY, T_saved ? T_saved : T16, dT16, dU, dV, dbias, colsum, accumulate, part, s);
}

// --------------------------------------- fp32, few rows, dimensions in whole tiles
// Two launches per direction: the slices of the rank-r intermediate, then every product that reads their sum.
static int linear_fwd_small(const pf_linear_desc *d, const LinearPlan &p, const float *X, const float *V, const float *U,
                            const float *bias, float *Y, float *T_save, Workspace &ws, hipStream_t s)
{
    const int M = (int)d->M, in = (int)d->in, out = (int)d->out, r = (int)d->r;
    float *P = ws.take<float>(p.n_small);
    const int S = linear_small_slices(in);
    int st = launch_ls_slices(s, "linear_T_slices", LsSliceArgs{X, V, P, in, r, M, in, r, S});
    if (st != PF_OK) return st;
    LsTileArgs ta = {};
    ls_add(ta, ls_operand(P, r, LS_MK, S, (i64)M * r), ls_operand(U, r, LS_MK), M, out, r, Y, out,
           d->has_bias ? bias : nullptr, 0, T_save);
    return launch_ls_tiles(s, "linear_Y=T*Ut+b", ta);
}

static int linear_bwd_small(const pf_linear_desc *d, const LinearPlan &p, const float *X, const float *V, const float *U,
                            const float *dY, const float *T_saved, float *dX, float *dU, float *dV, float *dbias,
                            int accumulate, Workspace &ws, hipStream_t s)
{
    const int M = (int)d->M, in = (int)d->in, out = (int)d->out, r = (int)d->r;
    float *PdT = ws.take<float>(p.n_small), *PT = ws.take<float>(p.n_small);
    const int SdT = linear_small_slices(out), ST = linear_small_slices(in);
    const bool recompute = dU && !T_saved;
    // dT = dY U in slices and, when T was not kept, T = X V again, in one launch
    int st = launch_ls_slices(s, "linear_dT_slices", LsSliceArgs{dY, U, PdT, out, r, M, out, r, SdT},
                              recompute ? LsSliceArgs{X, V, PT, in, r, M, in, r, ST} : LsSliceArgs{});
    if (st != PF_OK) return st;
    const LsOperand dT_rows = ls_operand(PdT, r, LS_MK, SdT, (i64)M * r); // (row, rank index)
    const LsOperand dT_cols = ls_operand(PdT, r, LS_KM, SdT, (i64)M * r); // (rank index, row): contraction over rows
    const bool want_db = d->has_bias && dbias;
    LsTileArgs ta = {};
    if (dX) ls_add(ta, dT_rows, ls_operand(V, r, LS_MK), M, in, r, dX, in, nullptr, 0);
    if (dU)
        ls_add(ta, ls_operand(dY, out, LS_KM), recompute ? ls_operand(PT, r, LS_KM, ST, (i64)M * r) : ls_operand(T_saved, r, LS_KM),
               out, r, M, dU, r, nullptr, accumulate, nullptr, want_db ? dbias : nullptr);
    else if (want_db) // only the bias gradient of this product is wanted: the column sums of its left operand
        ls_add(ta, ls_operand(dY, out, LS_KM), ls_operand(dY, out, LS_KM), out, 32, M, nullptr, 0, nullptr, accumulate, nullptr,
               dbias);
    if (dV) ls_add(ta, ls_operand(X, in, LS_KM), dT_cols, in, r, M, dV, r, nullptr, accumulate);
    return launch_ls_tiles(s, "linear_dX,dU,dV,db", ta);
}

// ------------------------------------------------------------- fp32, few rows
static int linear_T_skinny(const pf_linear_desc *d, const float *X, const float *V, float *T, float *part, hipStream_t s)
{
    const int M = (int)d->M, in = (int)d->in, r = (int)d->r;
    SkinnyArgs a;
    skinny_rows(M, X, in, V, r, in, r, part, a);
    int st = launch_skinny_gemm(s, "linear_T=X*V", a, false);
    if (st != PF_OK) return st;
    SliceSumArgs ss = {};
    ss.s[ss.nseg++] = skinny_rows_seg(a, M, T, a.p[0].N, nullptr);
    return launch_slice_sum(s, ss);
}

static int linear_fwd_skinny(const pf_linear_desc *d, const LinearPlan &p, const float *X, const float *V, const float *U,
                             const float *bias, float *Y, float *T_save, Workspace &ws, hipStream_t s)
{
    const int M = (int)d->M, out = (int)d->out, r = (int)d->r;
    float *Tws = ws.take<float>(p.n_T);
    float *part = ws.take<float>(p.n_part_sk);
    float *T = T_save ? T_save : Tws;
    int st = linear_T_skinny(d, X, V, T, part, s);
    if (st != PF_OK) return st;
    SkinnyArgs a;
    skinny_rows(M, T, r, U, r, r, out, part, a);
    st = launch_skinny_gemm(s, "linear_Y=T*Ut", a, true);
    if (st != PF_OK) return st;
    SliceSumArgs ss = {};
    ss.s[ss.nseg++] = skinny_rows_seg(a, M, Y, a.p[0].N, d->has_bias ? bias : nullptr);
    return launch_slice_sum(s, ss);
}

static int linear_bwd_skinny(const pf_linear_desc *d, const LinearPlan &p, const float *X, const float *V, const float *U,
                             const float *dY, const float *T_saved, float *dX, float *dU, float *dV, float *dbias,
                             int accumulate, Workspace &ws, hipStream_t s)
{
    const int M = (int)d->M, in = (int)d->in, out = (int)d->out, r = (int)d->r;
    float *Tws = ws.take<float>(p.n_T);
    float *dT = ws.take<float>(p.n_T);
    float *part = ws.take<float>(p.n_part_sk);
    int st = PF_OK;
    if (dU && !T_saved) { // T was not saved: recompute it
        st = linear_T_skinny(d, X, V, Tws, part, s);
        if (st != PF_OK) return st;
    }
    const float *T = T_saved ? T_saved : Tws;
    SkinnyArgs a;
    skinny_rows(M, dY, out, U, r, out, r, part, a);
    st = launch_skinny_gemm(s, "linear_dT=dY*U", a, false);
    if (st != PF_OK) return st;
    SliceSumArgs ss = {};
    ss.s[ss.nseg++] = skinny_rows_seg(a, M, dT, a.p[0].N, nullptr);
    st = launch_slice_sum(s, ss);
    if (st != PF_OK) return st;
    ss = SliceSumArgs{};
    if (dX) {
        skinny_rows(M, dT, r, V, r, r, in, part, a);
        st = launch_skinny_gemm(s, "linear_dX=dT*Vt", a, true);
        if (st != PF_OK) return st;
        ss.s[ss.nseg++] = skinny_rows_seg(a, M, dX, a.p[0].N, nullptr);
    }
    // factor gradients are rank-M updates; the slice sums of dX ride along
    RankArgs ra = {};
    ra.M = M;
    ra.accumulate = accumulate;
    rank_add(ra, dY, out, T, r, dU, r, out, r);
    rank_add(ra, X, in, dT, r, dV, r, in, r);
    if (d->has_bias && dbias) rank_add(ra, dY, out, nullptr, 0, dbias, 1, out, 1);
    return launch_rank_update(s, "linear_grads", ra, ss);
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

// ------------------------------------------------- projections that share their input
template <typename T>
__global__ void add_into_kernel(T *dst, const T *src, i64 count)
{
    const i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = from_float<T>(to_float(dst[i]) + to_float(src[i]));
}

template <typename T>
static int launch_add_into(hipStream_t s, T *dst, const T *src, i64 count)
{
    int st = PF_OK;
    if (count <= 0) return st;
    PF_LAUNCH(st, "add_into", add_into_kernel<T>, dim3((unsigned)((count + 255) / 256)), dim3(256), s, dst, src, count);
    return st;
}

struct SharedPlan {
    pf_linear_desc one; // one of the G layers
    LinearPlan p;
    bool fused_fwd, fused_bwd; // the groups run inside one launch of the chain kernel
    size_t n_colsum, fwd_bytes, bwd_bytes;
};

static int check_shared_desc(const pf_linear_shared_desc *d, pf_linear_desc *one)
{
    if (!d) return PF_ERR_NULL;
    *one = pf_linear_desc{d->M, d->n_in, d->n_out, d->r, d->dtype, PF_F32, d->has_bias};
    int st = check_linear_desc(one);
    if (st != PF_OK) return st;
    if (d->groups <= 0 || d->groups > 64) return PF_ERR_SHAPE;
    const i64 lim = 0x7fffffffLL;
    if (d->groups * d->M * d->n_out > (lim << 4)) return PF_ERR_SHAPE;
    return PF_OK;
}

static SharedPlan plan_shared(const pf_linear_shared_desc *d, const pf_linear_desc &one)
{
    SharedPlan sp;
    sp.one = one;
    sp.p = plan_linear(&one);
    const int G = d->groups;
    const bool bf = d->dtype == PF_BF16 && sp.p.chain2 && d->M > 0 && G > 1;
    sp.fused_fwd = bf && linear_chain2_multi_supported(d->n_in, d->n_out, d->r, G, false);
    sp.fused_bwd = bf && linear_chain2_multi_supported(d->n_out, d->n_in, d->r, G, true);
    sp.n_colsum = (size_t)(2 * ((d->M + LC_ROWS - 1) / LC_ROWS)) * d->n_out;
    const size_t el = d->dtype == PF_BF16 ? 2 : 4;
    sp.fwd_bytes = sp.p.fwd_bytes;
    // one layer's workspace, then: dT and (recomputed) T of all groups, their column sums, one more dX
    sp.bwd_bytes = sp.p.bwd_bytes + 2 * align_up((size_t)G * sp.p.n_T * 2) + align_up((size_t)G * sp.n_colsum * 4) +
                   align_up((size_t)(d->M * d->n_in) * el);
    return sp;
}

// Alignment a layer's slice of the stacked operands is held to: 16 bytes where the 16-byte-load kernels may run
// (their shapes make every slice a multiple of 16 bytes anyway), else that of an element or of the 4-byte loads
// of the few-row fp32 kernels.
static int layer_align(const SharedPlan &sp, size_t el) { return sp.p.fused ? 16 : (int)(el < 4 ? el : 4); }

template <typename T>
static int shared_bwd_loop(const pf_linear_shared_desc *d, const SharedPlan &sp, const T *X, const T *V, const T *U,
                           const T *dY, const T *T_saved, T *dX, float *dU, float *dV, float *dbias, int accumulate,
                           void *workspace, size_t workspace_bytes, hipStream_t s)
{
    // layer by layer; the input gradients of the layers after the first go to a spare buffer and are added
    const i64 M = d->M, in = d->n_in, out = d->n_out, r = d->r;
    T *spare = (T *)((char *)workspace + sp.p.bwd_bytes);
    int st = PF_OK;
    for (int g = 0; g < d->groups && st == PF_OK; ++g) {
        T *dXg = !dX ? nullptr : g == 0 ? dX : spare;
        st = linear_bwd_entry(&sp.one, X, V + g * in * r, U + g * out * r, dY + g * M * out,
                              T_saved ? T_saved + g * M * r : nullptr, dXg, dU ? dU + g * out * r : nullptr,
                              dV ? dV + g * in * r : nullptr, dbias ? dbias + g * out : nullptr, accumulate, workspace,
                              workspace_bytes, s, layer_align(sp, sizeof(T)));
        if (st == PF_OK && dX && g > 0) st = launch_add_into<T>(s, dX, spare, M * in);
    }
    return st;
}

} // namespace pf

using namespace pf;

// `align`: what the data pointers must be multiples of (16 for callers; the layers of a shared-input call may
// start anywhere an element does when their shape is one the element-wise kernels take)
int pf::linear_fwd_entry(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *bias,
                         void *Y, void *T_save, void *workspace, size_t workspace_bytes, void *stream, int align,
                         const LinEpilogue *ep)
{
    int st = check_linear_desc(d);
    if (st != PF_OK) return st;
    if (!V || !U || (d->has_bias && !bias)) return PF_ERR_NULL;
    if (d->M > 0 && (!X || !Y)) return PF_ERR_NULL;
    if (any_misaligned({X, V, U, bias, Y, T_save}, align)) return PF_ERR_UNSUPPORTED;
    const size_t need = plan_linear(d).fwd_bytes;
    if (need > 0 && (!workspace || workspace_bytes < need)) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    if (d->M == 0) return PF_OK;
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32 && plan_linear(d).small)
        return linear_fwd_small(d, plan_linear(d), (const float *)X, (const float *)V, (const float *)U,
                                (const float *)bias, (float *)Y, (float *)T_save, ws, s);
    if (d->dtype == PF_F32 && plan_linear(d).skinny)
        return linear_fwd_skinny(d, plan_linear(d), (const float *)X, (const float *)V, (const float *)U,
                                 (const float *)bias, (float *)Y, (float *)T_save, ws, s);
    if (d->dtype == PF_F32)
        return linear_fwd_generic<float>(d, (const float *)X, (const float *)V, (const float *)U, (const float *)bias,
                                         (float *)Y, (float *)T_save, ws, s);
    if (plan_linear(d).fused)
        return linear_fwd_fused(d, (const bf16_t *)X, (const bf16_t *)V, (const bf16_t *)U, (const bf16_t *)bias,
                                (bf16_t *)Y, (bf16_t *)T_save, ws, s, ep ? *ep : LinEpilogue{});
    return linear_fwd_generic<bf16_t>(d, (const bf16_t *)X, (const bf16_t *)V, (const bf16_t *)U,
                                      (const bf16_t *)bias, (bf16_t *)Y, (bf16_t *)T_save, ws, s);
}

int pf::linear_bwd_entry(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *dY,
                         const void *T_saved, void *dX, void *dU, void *dV, void *dbias, int accumulate,
                         void *workspace, size_t workspace_bytes, void *stream, int align, const LinEpilogue *ep)
{
    int st = check_linear_desc(d);
    if (st != PF_OK) return st;
    if (!V || !U) return PF_ERR_NULL;
    if (d->M > 0 && (!X || !dY)) return PF_ERR_NULL;
    if (any_misaligned({X, V, U, dY, T_saved, dX}, align) || any_misaligned({dU, dV, dbias}, 4)) return PF_ERR_UNSUPPORTED;
    const size_t need = plan_linear(d).bwd_bytes;
    if (need > 0 && (!workspace || workspace_bytes < need)) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32 && plan_linear(d).small)
        return linear_bwd_small(d, plan_linear(d), (const float *)X, (const float *)V, (const float *)U,
                                (const float *)dY, (const float *)T_saved, (float *)dX, (float *)dU, (float *)dV,
                                (float *)dbias, accumulate, ws, s);
    if (d->dtype == PF_F32 && plan_linear(d).skinny)
        return linear_bwd_skinny(d, plan_linear(d), (const float *)X, (const float *)V, (const float *)U,
                                 (const float *)dY, (const float *)T_saved, (float *)dX, (float *)dU, (float *)dV,
                                 (float *)dbias, accumulate, ws, s);
    if (d->dtype == PF_F32)
        return linear_bwd_generic<float>(d, (const float *)X, (const float *)V, (const float *)U, (const float *)dY,
                                         (const float *)T_saved, (float *)dX, (float *)dU, (float *)dV,
                                         (float *)dbias, accumulate, ws, s);
    const LinearPlan p = plan_linear(d);
    if (p.fused && dX && d->M > 0)
        return linear_bwd_fused(d, p, (const bf16_t *)X, (const bf16_t *)V, (const bf16_t *)U, (const bf16_t *)dY,
                                (const bf16_t *)T_saved, (bf16_t *)dX, (float *)dU, (float *)dV, (float *)dbias,
                                accumulate, ws, s, ep ? *ep : LinEpilogue{});
    return linear_bwd_generic<bf16_t>(d, (const bf16_t *)X, (const bf16_t *)V, (const bf16_t *)U,
                                      (const bf16_t *)dY, (const bf16_t *)T_saved, (bf16_t *)dX, (float *)dU,
                                      (float *)dV, (float *)dbias, accumulate, ws, s);
}

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
    return pf::linear_fwd_entry(d, X, V, U, bias, Y, T_save, workspace, workspace_bytes, stream, 16);
}

int pf_lowrank_linear_bwd(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *dY,
                          const void *T_saved, void *dX, void *dU, void *dV, void *dbias, int accumulate,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    return pf::linear_bwd_entry(d, X, V, U, dY, T_saved, dX, dU, dV, dbias, accumulate, workspace, workspace_bytes,
                                stream, 16);
}

} // extern "C"

// ---------------------------------------------------- library-owned scratch
// Backward for callers that cannot allocate: the partial sums of the factor gradients, the rank-r gradient dT
// and a recomputed T live in this array instead of a caller's workspace.  Every GPU the library runs on holds
// its own copy at its own address until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[PF_STATIC_SCRATCH_BYTES];

namespace pf {
constexpr int SCRATCH_MAX_DEVICES = 64;
static void *g_scratch_addr[SCRATCH_MAX_DEVICES]; // per device, looked up once
static std::mutex g_scratch_lock;

// Device address of `scratch` on the current device (no allocation: the array came with the code object).
static int scratch_on_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= SCRATCH_MAX_DEVICES)
        return set_hip_error(e != hipSuccess ? e : hipErrorInvalidDevice);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_addr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return set_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol);
        g_scratch_addr[dev] = ptr;
    }
    *out = g_scratch_addr[dev];
    return PF_OK;
}
} // namespace pf

extern "C" {

size_t pf_static_scratch_bytes(void) { return (size_t)PF_STATIC_SCRATCH_BYTES; }

int pf_lowrank_linear_bwd_static(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *dY,
                                 const void *T_saved, void *dX, void *dU, void *dV, void *dbias, int accumulate,
                                 void *stream)
{
    int st = check_linear_desc(d);
    if (st != PF_OK) return st;
    if (plan_linear(d).bwd_bytes > (size_t)PF_STATIC_SCRATCH_BYTES) return PF_ERR_WORKSPACE;
    void *ptr = nullptr;
    st = scratch_on_current_device(&ptr);
    if (st != PF_OK) return st;
    // nothing in the backward pass reads scratch memory before writing it, so what the last call left is harmless
    return pf::linear_bwd_entry(d, X, V, U, dY, T_saved, dX, dU, dV, dbias, accumulate, ptr,
                                (size_t)PF_STATIC_SCRATCH_BYTES, stream, 16);
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
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32)
        return dense_linear_bwd_t<float>(d, (const float *)X, (const float *)W, (const float *)dY, (float *)dX,
                                         (float *)dW, (float *)dbias, accumulate, ws, s);
    return dense_linear_bwd_t<bf16_t>(d, (const bf16_t *)X, (const bf16_t *)W, (const bf16_t *)dY, (bf16_t *)dX,
                                      (float *)dW, (float *)dbias, accumulate, ws, s);
}

size_t pf_lowrank_linear_shared_fwd_workspace_bytes(const pf_linear_shared_desc *d)
{
    pf_linear_desc one;
    if (check_shared_desc(d, &one) != PF_OK) return 0;
    return plan_shared(d, one).fwd_bytes;
}

size_t pf_lowrank_linear_shared_bwd_workspace_bytes(const pf_linear_shared_desc *d)
{
    pf_linear_desc one;
    if (check_shared_desc(d, &one) != PF_OK) return 0;
    return plan_shared(d, one).bwd_bytes;
}

int pf_lowrank_linear_shared_fwd(const pf_linear_shared_desc *d, const void *X, const void *V, const void *U,
                                 const void *bias, void *Y, void *T_save, void *workspace, size_t workspace_bytes,
                                 void *stream)
{
    pf_linear_desc one;
    int st = check_shared_desc(d, &one);
    if (st != PF_OK) return st;
    if (!V || !U || (d->has_bias && !bias)) return PF_ERR_NULL;
    if (d->M > 0 && (!X || !Y)) return PF_ERR_NULL;
    if (any_misaligned({X, V, U, bias, Y, T_save}, 16)) return PF_ERR_UNSUPPORTED;
    const SharedPlan sp = plan_shared(d, one);
    if (sp.fwd_bytes > 0 && (!workspace || workspace_bytes < sp.fwd_bytes)) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    if (d->M == 0) return PF_OK;
    const i64 M = d->M, in = d->n_in, out = d->n_out, r = d->r;
    hipStream_t s = (hipStream_t)stream;
    if (sp.fused_fwd) {
        LinChainArgs c{(const uint16_t *)X, (const uint16_t *)V, (const uint16_t *)U,
                       d->has_bias ? (const uint16_t *)bias : nullptr, (uint16_t *)Y, (uint16_t *)T_save, nullptr,
                       M, (int)in, (int)out};
        c.groups = d->groups;
        c.gs_W1 = in * r;
        c.gs_W2 = out * r;
        c.gs_bias = out;
        c.gs_out = M * out;
        c.gs_mid = M * r;
        return launch_linear_chain2(s, "linear_shared_fwd_fused", c);
    }
    const size_t el = d->dtype == PF_BF16 ? 2 : 4;
    for (int g = 0; g < d->groups && st == PF_OK; ++g)
        st = linear_fwd_entry(&one, X, (const char *)V + g * in * r * el, (const char *)U + g * out * r * el,
                              bias ? (const char *)bias + g * out * el : nullptr, (char *)Y + g * M * out * el,
                              T_save ? (char *)T_save + g * M * r * el : nullptr, workspace, workspace_bytes, stream,
                              layer_align(sp, el));
    return st;
}

int pf_lowrank_linear_shared_bwd(const pf_linear_shared_desc *d, const void *X, const void *V, const void *U,
                                 const void *dY, const void *T_saved, void *dX, void *dU, void *dV, void *dbias,
                                 int accumulate, void *workspace, size_t workspace_bytes, void *stream)
{
    pf_linear_desc one;
    int st = check_shared_desc(d, &one);
    if (st != PF_OK) return st;
    if (!V || !U) return PF_ERR_NULL;
    if (d->M > 0 && (!X || !dY)) return PF_ERR_NULL;
    if (any_misaligned({X, V, U, dY, T_saved, dX}, 16) || any_misaligned({dU, dV, dbias}, 4)) return PF_ERR_UNSUPPORTED;
    const SharedPlan sp = plan_shared(d, one);
    if (!workspace || workspace_bytes < sp.bwd_bytes) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    hipStream_t s = (hipStream_t)stream;
    const i64 M = d->M, in = d->n_in, out = d->n_out, r = d->r;
    const int G = d->groups;
    if (!(sp.fused_bwd && dX)) {
        if (d->dtype == PF_F32)
            return shared_bwd_loop<float>(d, sp, (const float *)X, (const float *)V, (const float *)U, (const float *)dY,
                                          (const float *)T_saved, (float *)dX, (float *)dU, (float *)dV,
                                          (float *)dbias, accumulate, workspace, workspace_bytes, s);
        return shared_bwd_loop<bf16_t>(d, sp, (const bf16_t *)X, (const bf16_t *)V, (const bf16_t *)U,
                                       (const bf16_t *)dY, (const bf16_t *)T_saved, (bf16_t *)dX, (float *)dU,
                                       (float *)dV, (float *)dbias, accumulate, workspace, workspace_bytes, s);
    }
    // fused: every group's dT = dY_g U_g and the sum dX = sum_g dT_g V_g^T in one launch, then the factor
    // gradients layer by layer
    Workspace ws(workspace, workspace_bytes);
    const size_t grads = (size_t)sp.p.wg_groups * r * (in + out);
    float *part = ws.take<float>(grads > sp.p.n_part ? grads : sp.p.n_part);
    bf16_t *dT16 = ws.take<bf16_t>((size_t)G * sp.p.n_T);
    bf16_t *T16 = ws.take<bf16_t>((size_t)G * sp.p.n_T);
    float *colsum = ws.take<float>((size_t)G * sp.n_colsum);
    const bool want_db = d->has_bias && dbias;
    const bf16_t *Xb = (const bf16_t *)X, *Vb = (const bf16_t *)V, *Ub = (const bf16_t *)U, *dYb = (const bf16_t *)dY;
    const bf16_t *Tb = (const bf16_t *)T_saved;
    if (dU && !Tb) { // T was not saved: recompute it
        for (int g = 0; g < G && st == PF_OK; ++g)
            st = launch_gemm_generic<bf16_t, true, false>(
                "linear_T=X*V", s, GemmShape{(int)M, (int)r, (int)in, 1, 1}, OpA_RowMajor<bf16_t>{Xb, (int)in, 0},
                OpB_KN<bf16_t>{Vb + g * in * r, (int)r, 0, 0},
                EpiRowMajor<bf16_t, bf16_t>{T16 + g * M * r, nullptr, (int)r, nullptr, 0});
        if (st != PF_OK) return st;
        Tb = T16;
    }
    LinChainArgs c{(const uint16_t *)dYb, (const uint16_t *)Ub, (const uint16_t *)Vb, nullptr, (uint16_t *)dX,
                   (uint16_t *)dT16, want_db ? colsum : nullptr, M, (int)out, (int)in};
    c.groups = G;
    c.sum_out = 1;
    c.gs_in = M * out;
    c.gs_W1 = out * r;
    c.gs_W2 = in * r;
    c.gs_mid = M * r;
    c.gs_colsum = (i64)sp.n_colsum;
    st = launch_linear_chain2(s, "linear_shared_bwd_data_fused", c);
    for (int g = 0; g < G && st == PF_OK; ++g)
        st = linear_wgrads_fused(&one, sp.p, Xb, dYb + g * M * out, Tb ? Tb + g * M * r : nullptr, dT16 + g * M * r,
                                 dU ? (float *)dU + g * out * r : nullptr, dV ? (float *)dV + g * in * r : nullptr,
                                 dbias ? (float *)dbias + g * out : nullptr, want_db ? colsum + g * sp.n_colsum : nullptr,
                                 accumulate, part, s);
    return st;
}

} // extern "C"

// ------------------------------------------------ entry points with an epilogue
// (the element-wise part is applied by the caller when *fused stays false)
int pf::linear_fwd_entry_ep(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *bias,
                            const void *residual, int act, void *Y, void *T_save, void *workspace,
                            size_t workspace_bytes, void *stream, bool *fused)
{
    *fused = false;
    const LinEpilogue ep{residual, nullptr, act == PF_ACT_RELU ? 1 : 0, fused};
    return pf::linear_fwd_entry(d, X, V, U, bias, Y, T_save, workspace, workspace_bytes, stream, 16, &ep);
}

int pf::linear_bwd_entry_ep(const pf_linear_desc *d, const void *X, const void *V, const void *U, const void *dZ,
                            const void *T_saved, const void *dX_add, int x_is_relu, void *dX, void *dU, void *dV,
                            void *dbias, int accumulate, void *workspace, size_t workspace_bytes, void *stream,
                            bool *fused)
{
    *fused = false;
    const LinEpilogue ep{dX_add, x_is_relu ? X : nullptr, 0, fused};
    return pf::linear_bwd_entry(d, X, V, U, dZ, T_saved, dX, dU, dV, dbias, accumulate, workspace, workspace_bytes,
                                stream, 16, &ep);
}
