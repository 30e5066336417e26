// Factorized convolution (paper Section 2.2): thin k x k convolution into r channels
// followed by a 1x1 convolution, forward and backward, plus the dense comparator.
// Host-side validation, workspace planning and dispatch; the any-shape path runs every
// stage as an implicit GEMM (operands gathered by functors) on the guarded tile GEMM.
#include "pf_conv_chain.h"
#include "pf_conv_wgrad.h"
#include "pf_epilogue.h"

namespace pf {

struct ConvGeom {
    int N, C, H, W, Cout, r, k, s, p, Ho, Wo;
};

// B(kidx = (c,i,j), n = (img,y,x)) = Xpad[img, c, y s + i - p, x s + j - p]
template <typename T>
struct OpB_Im2col {
    const T *X;
    ConvGeom g;
    __device__ __forceinline__ float at(int kidx, int n) const
    {
        const int kk = g.k * g.k;
        const int c = kidx / kk, t = kidx % kk, i = t / g.k, j = t % g.k;
        const int hw = g.Ho * g.Wo;
        const int img = n / hw, pix = n % hw, y = pix / g.Wo, x = pix % g.Wo;
        const int yy = y * g.s + i - g.p, xx = x * g.s + j - g.p;
        if (yy < 0 || yy >= g.H || xx < 0 || xx >= g.W) return 0.f;
        return to_float(X[(((i64)img * g.C + c) * g.H + yy) * g.W + xx]);
    }
    __device__ __forceinline__ float operator()(int k, int n, int) const { return at(k, n); }
};
// B(k = (img,y,x), n = (c,i,j)): the same view with the roles swapped (weight gradient)
template <typename T>
struct OpB_Im2colT {
    OpB_Im2col<T> v;
    __device__ __forceinline__ float operator()(int k, int n, int) const { return v.at(n, k); }
};

// Tensor P[img, ch, pix] (NCHW with HW flattened) seen as a matrix over (channel, pixel).
template <typename T>
struct OpB_NCHW { // B(k = ch, n = (img,pix))
    const T *p;
    int CH, HW;
    __device__ __forceinline__ float operator()(int k, int n, int) const
    {
        const int img = n / HW, pix = n % HW;
        return to_float(p[((i64)img * CH + k) * HW + pix]);
    }
};
template <typename T>
struct OpB_NCHW_T { // B(k = (img,pix), n = ch)
    const T *p;
    int CH, HW;
    __device__ __forceinline__ float operator()(int k, int n, int) const
    {
        const int img = k / HW, pix = k % HW;
        return to_float(p[((i64)img * CH + n) * HW + pix]);
    }
};
template <typename T>
struct OpA_NCHW { // A(m = ch, k = (img,pix))
    const T *p;
    int CH, HW;
    __device__ __forceinline__ float operator()(int m, int k, int) const
    {
        const int img = k / HW, pix = k % HW;
        return to_float(p[((i64)img * CH + m) * HW + pix]);
    }
};

// A(m = c, kidx = (q,i,j)) = Uk[q, c, i, j]
template <typename T>
struct OpA_FilterT {
    const T *Uk;
    int C, kk;
    __device__ __forceinline__ float operator()(int m, int kidx, int) const
    {
        const int q = kidx / kk, t = kidx % kk;
        return to_float(Uk[((i64)q * C + m) * kk + t]);
    }
};

// B(kidx = (q,i,j), n = (img,yy,xx)) = dT[img, q, y, x] where y s + i - p = yy, x s + j - p = xx
template <typename T>
struct OpB_Col2im {
    const T *dT;
    ConvGeom g;
    int CH; // channels of dT
    __device__ __forceinline__ float operator()(int kidx, int n, int) const
    {
        const int kk = g.k * g.k;
        const int q = kidx / kk, t = kidx % kk, i = t / g.k, j = t % g.k;
        const int hw = g.H * g.W;
        const int img = n / hw, pix = n % hw, yy = pix / g.W, xx = pix % g.W;
        const int ys = yy + g.p - i, xs = xx + g.p - j;
        if (ys < 0 || xs < 0 || ys % g.s || xs % g.s) return 0.f;
        const int y = ys / g.s, x = xs / g.s;
        if (y >= g.Ho || x >= g.Wo) return 0.f;
        return to_float(dT[(((i64)img * CH + q) * g.Ho + y) * g.Wo + x]);
    }
};

// C(m = ch, n = (img,pix)) -> P[img, ch, pix], optionally to a second buffer
template <typename T1, typename T2>
struct EpiNCHW {
    T1 *c1;
    T2 *c2;
    int CH, HW;
    __device__ __forceinline__ void operator()(int m, int n, float acc, int, int) const
    {
        const int img = n / HW, pix = n % HW;
        const i64 off = ((i64)img * CH + m) * HW + pix;
        if (c1) c1[off] = from_float<T1>(acc);
        if (c2) c2[off] = from_float<T2>(acc);
    }
};

// ------------------------------------------------------------ validation
static int check_conv_desc(const pf_conv_desc *d, ConvGeom *g)
{
    if (!d) return PF_ERR_NULL;
    if (d->dtype != PF_F32 && d->dtype != PF_BF16) return PF_ERR_UNSUPPORTED;
    if (d->layout != PF_NCHW || d->wgrad_dtype != PF_F32) return PF_ERR_UNSUPPORTED;
    if (d->N < 0 || d->Cin <= 0 || d->H <= 0 || d->W <= 0 || d->Cout <= 0 || d->r <= 0) return PF_ERR_SHAPE;
    if (d->k <= 0 || d->stride <= 0 || d->pad < 0 || d->k > 15) return PF_ERR_SHAPE;
    const i64 Ho = (d->H + 2 * (i64)d->pad - d->k) / d->stride + 1, Wo = (d->W + 2 * (i64)d->pad - d->k) / d->stride + 1;
    if (d->H + 2 * (i64)d->pad < d->k || d->W + 2 * (i64)d->pad < d->k || Ho <= 0 || Wo <= 0) return PF_ERR_SHAPE;
    const i64 lim = 0x7fffffffLL;
    if (d->N * d->H * d->W > lim || d->N * Ho * Wo > lim || d->Cin * d->k * d->k > lim || d->r * d->k * d->k > lim ||
        d->Cout > lim || d->r > lim)
        return PF_ERR_SHAPE;
    if (d->N * d->Cin * d->H * d->W > (lim << 4) || d->N * d->Cout * Ho * Wo > (lim << 4)) return PF_ERR_SHAPE;
    if (g) *g = ConvGeom{(int)d->N, (int)d->Cin, (int)d->H, (int)d->W, (int)d->Cout, (int)d->r,
                         d->k,      d->stride,   d->pad,    (int)Ho,   (int)Wo};
    return PF_OK;
}

struct ConvPlan {
    int ks_dVp, ks_dUk;
    size_t n_T, n_part, fwd_bytes, bwd_bytes;
    bool chain;              // the fused small-image kernel applies (bf16 only)
    bool wgrad;              // the small-image filter-gradient kernel applies (bf16 only)
    int wg_groups, wg_ipg;   // image groups and images per group of that kernel, k x k stage
    int wg_groups2, wg_ipg2; // the same for the 1x1 stage
    size_t n_w1, n_w2;       // packed weight elements, forward direction
    size_t n_w1b, n_w2b;     // packed weight elements, backward direction
    size_t saved_bytes;      // the backward direction's packed weights when the forward call saves them
};

static ConvPlan plan_conv(const ConvGeom &g, int dtype)
{
    ConvPlan p;
    p.chain = dtype == PF_BF16 && chain_supported(g.C, g.Cout, g.r, g.H, g.W, g.k, g.s, g.p);
    p.n_w1 = chain_w1_elems(g.C, g.r, g.k);
    p.n_w2 = chain_w2_elems(g.Cout, g.r, 1);
    p.n_w1b = chain_w1_elems(g.Cout, g.r, 1);
    p.n_w2b = chain_w2_elems(g.C, g.r, g.k);
    p.saved_bytes = p.chain ? align_up(p.n_w1b * 2) + align_up(p.n_w2b * 2) : 0;
    p.wgrad = p.chain && wgrad_supported(g.r, g.C, g.H, g.W, g.k, g.s, g.p) &&
              wgrad_supported(g.r, g.Cout, g.H, g.W, 1, 1, 0);
    p.wg_groups = p.wg_ipg = p.wg_groups2 = p.wg_ipg2 = 1;
    if (p.wgrad && g.N > 0) {
        // Image groups of the two problems of the launch.  A problem has `units` independent output blocks;
        // with g groups it runs units * g workgroups of ceil(N / g) images each and writes g partial sums.  Both
        // problems should fit the chip in one round (one workgroup per compute unit) and finish together, and
        // every extra group costs a partial sum to write and to add up.  Costs in thousands of cycles, from
        // traces of the kernel: an image of a 3x3 block 0.7 (rank 64) or 1.4, of a 1x1 block 1.0 (rank 64) or 2.0;
        // a megabyte of partial sums 1.0.  The search is tiny: every g1, and for it the fewest groups g2 that
        // do not make problem 2 the longer one.
        const int units1 = (g.C / wgrad_nchunk(g.r, g.k, 1)) * (g.k == 3 ? 2 : 1);
        const int units2 = g.Cout / wgrad_nchunk(g.r, 1, 2);
        const double c1 = g.k == 3 ? (g.r == 128 ? 1.4 : 0.7) : g.r == 128 ? 2.0 : 1.0, c2 = g.r == 128 ? 2.0 : 1.0;
        const double mb1 = 1.0e-6 * 4.0 * g.r * g.C * g.k * g.k, mb2 = 1.0e-6 * 4.0 * g.r * g.Cout;
        const int budget = 256;
        double best = 1e30;
        for (int g1 = 1; g1 <= g.N && (g1 == 1 || units1 * g1 + units2 <= budget); ++g1) {
            const int ipg1 = (g.N + g1 - 1) / g1;
            int g2max = (budget - units1 * g1) / units2;
            g2max = g2max < 1 ? 1 : g2max > g.N ? g.N : g2max;
            int ipg2 = (int)(ipg1 * c1 / c2); // images a workgroup of problem 2 may take
            ipg2 = ipg2 < 1 ? 1 : ipg2;
            int g2 = (g.N + ipg2 - 1) / ipg2;
            g2 = g2 > g2max ? g2max : g2;
            ipg2 = (g.N + g2 - 1) / g2;
            const double t1 = ipg1 * c1, t2 = ipg2 * c2;
            const double t = (t1 > t2 ? t1 : t2) + g1 * mb1 + g2 * mb2;
            if (t < best) {
                best = t;
                p.wg_ipg = ipg1;
                p.wg_ipg2 = ipg2;
            }
        }
        p.wg_groups = (g.N + p.wg_ipg - 1) / p.wg_ipg;
        p.wg_groups2 = (g.N + p.wg_ipg2 - 1) / p.wg_ipg2;
    }
    const i64 npix = (i64)g.N * g.Ho * g.Wo;
    p.ks_dVp = choose_ksplit(g.Cout, g.r, npix);
    p.ks_dUk = choose_ksplit(g.r, (i64)g.C * g.k * g.k, npix);
    p.n_T = (size_t)(npix * g.r);
    size_t a = (size_t)p.ks_dVp * g.Cout * g.r, b = (size_t)p.ks_dUk * g.r * g.C * g.k * g.k;
    p.n_part = a > b ? a : b;
    if (p.wgrad) { // both partial sets live side by side
        const size_t both = (size_t)p.wg_groups2 * g.Cout * g.r + (size_t)p.wg_groups * g.r * g.C * g.k * g.k;
        if (both > p.n_part) p.n_part = both;
    }
    p.fwd_bytes = align_up(p.n_T * sizeof(float));
    p.bwd_bytes = 2 * align_up(p.n_T * sizeof(float)) + align_up(p.n_part * sizeof(float));
    if (p.chain) { // the fused path needs packed weights instead of float copies of T (take the larger)
        const size_t f = align_up(p.n_w1 * 2) + align_up(p.n_w2 * 2);
        const size_t b = align_up(p.n_w1b * 2) + align_up(p.n_w2b * 2) + 2 * align_up(p.n_T * 2) +
                         align_up(p.n_part * sizeof(float));
        if (f > p.fwd_bytes) p.fwd_bytes = f;
        if (b > p.bwd_bytes) p.bwd_bytes = b;
    }
    return p;
}

// ------------------------------------------------------------- any-shape
template <typename T>
static int conv_T_generic(const ConvGeom &g, const T *X, const T *Uk, float *Tws, T *T_save, hipStream_t s)
{
    const int npix = g.N * g.Ho * g.Wo, K = g.C * g.k * g.k;
    return launch_gemm_generic<T, true, false>("conv_T=Uk*X", s, GemmShape{g.r, npix, K, 1, 1},
                                               OpA_RowMajor<T>{Uk, K, 0}, OpB_Im2col<T>{X, g},
                                               EpiNCHW<float, T>{Tws, T_save, g.r, g.Ho * g.Wo});
}

template <typename T>
static int conv_fwd_generic(const ConvGeom &g, const T *X, const T *Uk, const T *Vp, T *Y, T *T_save, Workspace &ws,
                            hipStream_t s)
{
    const int npix = g.N * g.Ho * g.Wo;
    float *Tws = ws.take<float>((size_t)npix * g.r);
    int st = conv_T_generic<T>(g, X, Uk, Tws, T_save, s);
    if (st != PF_OK) return st;
    return launch_gemm_generic<T, true, false>("conv_Y=Vp*T", s, GemmShape{g.Cout, npix, g.r, 1, 1},
                                               OpA_RowMajor<T>{Vp, g.r, 0}, OpB_NCHW<float>{Tws, g.r, g.Ho * g.Wo},
                                               EpiNCHW<T, T>{Y, nullptr, g.Cout, g.Ho * g.Wo});
}

// Filter gradients from the saved / recomputed T and from dT (both [N][r][pixels], any element type).
template <typename T, typename TT, typename TD>
static int conv_wgrads(const ConvGeom &g, const ConvPlan &p, const T *X, const T *dY, const TT *Tt, const TD *dT,
                       float *dUk, float *dVp, int accumulate, float *part, hipStream_t s)
{
    const int npix = g.N * g.Ho * g.Wo, HW = g.Ho * g.Wo, kk = g.k * g.k;
    int st = PF_OK;
    if (dVp) { // dVp[o,q] = sum_pixel dY[o,pixel] T[q,pixel]
        st = launch_gemm_generic<T, true, true>("conv_dVp=dY*Tt", s, GemmShape{g.Cout, g.r, npix, 1, p.ks_dVp},
                                                OpA_NCHW<T>{dY, g.Cout, HW}, OpB_NCHW_T<TT>{Tt, g.r, HW},
                                                EpiPartial{part, g.r, (i64)g.Cout * g.r});
        if (st == PF_OK) st = launch_splitk_reduce(s, part, dVp, (i64)g.Cout * g.r, p.ks_dVp, accumulate);
        if (st != PF_OK) return st;
    }
    if (dUk) { // dUk[q,(c,i,j)] = sum_pixel dT[q,pixel] Xcol[(c,i,j),pixel]
        st = launch_gemm_generic<T, true, true>("conv_dUk=dT*Xcolt", s, GemmShape{g.r, g.C * kk, npix, 1, p.ks_dUk},
                                                OpA_NCHW<TD>{dT, g.r, HW}, OpB_Im2colT<T>{OpB_Im2col<T>{X, g}},
                                                EpiPartial{part, (i64)g.C * kk, (i64)g.r * g.C * kk});
        if (st == PF_OK) st = launch_splitk_reduce(s, part, dUk, (i64)g.r * g.C * kk, p.ks_dUk, accumulate);
    }
    return st;
}

template <typename T>
static int conv_bwd_generic(const ConvGeom &g, const ConvPlan &p, const T *X, const T *Uk, const T *Vp, const T *dY,
                            const T *T_saved, T *dX, float *dUk, float *dVp, int accumulate, Workspace &ws,
                            hipStream_t s)
{
    const int npix = g.N * g.Ho * g.Wo, HW = g.Ho * g.Wo, kk = g.k * g.k;
    float *Tws = ws.take<float>(p.n_T);
    float *dTws = ws.take<float>(p.n_T);
    float *part = ws.take<float>(p.n_part);
    int st = PF_OK;
    if (dVp && !T_saved) {
        st = conv_T_generic<T>(g, X, Uk, Tws, nullptr, s);
        if (st != PF_OK) return st;
    }
    if (dX || dUk) { // dT[q, pixel] = sum_o Vp[o,q] dY[o, pixel]
        st = launch_gemm_generic<T, false, false>("conv_dT=Vpt*dY", s, GemmShape{g.r, npix, g.Cout, 1, 1},
                                                  OpA_ColMajor<T>{Vp, g.r, 0}, OpB_NCHW<T>{dY, g.Cout, HW},
                                                  EpiNCHW<float, float>{dTws, nullptr, g.r, HW});
        if (st != PF_OK) return st;
    }
    if (dX) { // dX[c, in-pixel] = sum_{q,i,j} Uk[q,c,i,j] dT[q, out-pixel(in-pixel,i,j)]
        st = launch_gemm_generic<T, true, false>("conv_dX=Ukt*dT", s, GemmShape{g.C, g.N * g.H * g.W, g.r * kk, 1, 1},
                                                 OpA_FilterT<T>{Uk, g.C, kk}, OpB_Col2im<float>{dTws, g, g.r},
                                                 EpiNCHW<T, T>{dX, nullptr, g.C, g.H * g.W});
        if (st != PF_OK) return st;
    }
    if (T_saved) return conv_wgrads<T, T, float>(g, p, X, dY, T_saved, dTws, dUk, dVp, accumulate, part, s);
    return conv_wgrads<T, float, float>(g, p, X, dY, Tws, dTws, dUk, dVp, accumulate, part, s);
}

// ----------------------------------------------------- fused small-image path (bf16)
// What the chain kernel applies as it stores its output (all optional): forward scale / shift / residual / ReLU,
// backward the gradient arriving over a skip connection and the mask of a ReLU input.
struct ConvEpilogue {
    const float *scale, *shift;
    const void *add, *mask;
    int relu;
};

static int conv_fwd_chain(const ConvGeom &g, const ConvPlan &p, const bf16_t *X, const bf16_t *Uk, const bf16_t *Vp,
                          bf16_t *Y, bf16_t *T_save, void *W_save, Workspace &ws, hipStream_t s, const ConvEpilogue &ep)
{
    const int T = g.k * g.k;
    uint16_t *w1 = ws.take<uint16_t>(p.n_w1);
    uint16_t *w2 = ws.take<uint16_t>(p.n_w2);
    // Both factors are re-ordered into MFMA fragment order by one small launch (read in place, one lane per row,
    // the 1x1 filters Vp[Cout][r] reach the compute unit at a quarter of the rate).  The same launch can re-order
    // both factors the way the backward pass wants them (W_save), which saves that pass a launch of its own.
    uint16_t *s1 = (uint16_t *)W_save, *s2 = W_save ? (uint16_t *)((char *)W_save + align_up(p.n_w1b * 2)) : nullptr;
    int st = launch_pack_chain(
        s, make_pack_w1((const uint16_t *)Uk, (uint4 *)w1, g.C, g.r, g.k, (i64)g.C * T, T, 1, g.H, g.W),
        make_pack_w2(W_save ? (const uint16_t *)Uk : nullptr, (uint4 *)s2, g.C, g.r, g.k, T - 1, T, (i64)g.C * T, -1),
        // (kept for a backward call that is given the same scale: its first stage runs on scale * Vp)
        [&] {
            PackW1 q = make_pack_w1(W_save ? (const uint16_t *)Vp : nullptr, (uint4 *)s1, g.Cout, g.r, 1, 1, g.r, 0, g.H, g.W);
            q.cscale = ep.scale;
            return q;
        }(),
        make_pack_w2((const uint16_t *)Vp, (uint4 *)w2, g.Cout, g.r, 1, 0, g.r, 1, 0));
    if (st != PF_OK) return st;
    ChainArgs a{(const uint16_t *)X, (const uint4 *)w1, (const uint4 *)w2, nullptr, (uint16_t *)Y,
                (uint16_t *)T_save,  g.C,               g.Cout,            g.H,     g.W,
                0,                   nullptr,           ep.scale,          ep.shift, (const uint16_t *)ep.add,
                (const uint16_t *)ep.mask, ep.relu};
    return launch_conv_chain(s, "conv_fwd_fused", a, g.N, g.k, 1, g.r);
}

static int conv_bwd_chain(const ConvGeom &g, const ConvPlan &p, const bf16_t *X, const bf16_t *Uk, const bf16_t *Vp,
                          const bf16_t *dY, const bf16_t *T_saved, const void *W_saved, bf16_t *dX, float *dUk,
                          float *dVp, int accumulate, Workspace &ws, hipStream_t s, const ConvEpilogue &ep)
{
    const int T = g.k * g.k;
    const uint16_t *w1 = ws.take<uint16_t>(p.n_w1b);
    const uint16_t *w2 = ws.take<uint16_t>(p.n_w2b);
    if (W_saved) { // the forward call packed them already
        w1 = (const uint16_t *)W_saved;
        w2 = (const uint16_t *)((const char *)W_saved + align_up(p.n_w1b * 2));
    }
    bf16_t *dT16 = ws.take<bf16_t>(p.n_T);
    bf16_t *T16 = ws.take<bf16_t>(p.n_T);
    float *part = ws.take<float>(p.n_part);
    int st = PF_OK;
    if (dVp && !T_saved) { // T was not saved: recompute it (thin convolution only)
        st = launch_gemm_generic<bf16_t, true, false>(
            "conv_T=Uk*X", s, GemmShape{g.r, g.N * g.Ho * g.Wo, g.C * T, 1, 1}, OpA_RowMajor<bf16_t>{Uk, (i64)g.C * T, 0},
            OpB_Im2col<bf16_t>{X, g}, EpiNCHW<bf16_t, bf16_t>{T16, nullptr, g.r, g.Ho * g.Wo});
        if (st != PF_OK) return st;
    }
    // stage 1: dT = Vp^T dY (1x1); stage 2: dX = flipped-Uk * dT (k x k)
    if (!W_saved) {
        PackW1 q = make_pack_w1((const uint16_t *)Vp, (uint4 *)w1, g.Cout, g.r, 1, 1, g.r, 0, g.H, g.W);
        q.cscale = ep.scale; // dT = Vp^T (scale dZ) = (scale Vp)^T dZ
        st = launch_pack_chain(s, q, make_pack_w2((const uint16_t *)Uk, (uint4 *)w2, g.C, g.r, g.k, T - 1, T, (i64)g.C * T, -1));
    }
    if (st != PF_OK) return st;
    ChainArgs a{(const uint16_t *)dY, (const uint4 *)w1, (const uint4 *)w2, nullptr, (uint16_t *)dX,
                (uint16_t *)dT16,     g.Cout,            g.C,               g.H,     g.W,
                0,                    nullptr,           nullptr,           nullptr, (const uint16_t *)ep.add,
                (const uint16_t *)ep.mask, 0};
    st = launch_conv_chain(s, "conv_bwd_data_fused", a, g.N, 1, g.k, g.r);
    if (st != PF_OK) return st;
    const bf16_t *Tt = T_saved ? T_saved : T16;
    if (!p.wgrad) return conv_wgrads<bf16_t, bf16_t, bf16_t>(g, p, X, dY, Tt, dT16, dUk, dVp, accumulate, part, s);
    float *part_dUk = part, *part_dVp = part + (size_t)p.wg_groups * g.r * g.C * T;
    WgradArgs wa1{(const uint16_t *)dT16, (const uint16_t *)X, dUk ? part_dUk : nullptr, g.r, g.C, g.H, g.W, g.N,
                  p.wg_ipg,               p.wg_groups, 0};
    WgradArgs wa2{(const uint16_t *)Tt, (const uint16_t *)dY, dVp ? part_dVp : nullptr, g.r, g.Cout, g.H, g.W, g.N,
                  p.wg_ipg2,            p.wg_groups2, 0};
    st = launch_conv_wgrad_pair(s, wa1, g.k, wa2);
    if (st != PF_OK) return st;
    WgradReduceArgs r0{part_dUk, dUk, p.wg_groups, T, g.r, g.C, (i64)g.C * T, T, 1, accumulate, nullptr};
    WgradReduceArgs r1{part_dVp, dVp, p.wg_groups2, 1, g.r, g.Cout, 1, g.r, 0, accumulate, ep.scale}; // dVp = scale (dZ T^T)
    return launch_wgrad_reduce(s, r0, r1);
}

// ------------------------------------------------------------------ dense
struct DenseConvPlan {
    int ks;
    size_t n_part, bytes;
};
static DenseConvPlan plan_dense_conv(const ConvGeom &g)
{
    DenseConvPlan p;
    const i64 npix = (i64)g.N * g.Ho * g.Wo;
    p.ks = choose_ksplit(g.Cout, (i64)g.C * g.k * g.k, npix);
    p.n_part = (size_t)p.ks * g.Cout * g.C * g.k * g.k;
    p.bytes = align_up(p.n_part * sizeof(float));
    return p;
}

template <typename T>
static int dense_conv_fwd_t(const ConvGeom &g, const T *X, const T *Wd, T *Y, hipStream_t s)
{
    const int npix = g.N * g.Ho * g.Wo, K = g.C * g.k * g.k;
    return launch_gemm_generic<T, true, false>("dense_conv_Y=W*X", s, GemmShape{g.Cout, npix, K, 1, 1},
                                               OpA_RowMajor<T>{Wd, K, 0}, OpB_Im2col<T>{X, g},
                                               EpiNCHW<T, T>{Y, nullptr, g.Cout, g.Ho * g.Wo});
}

template <typename T>
static int dense_conv_bwd_t(const ConvGeom &g, const T *X, const T *Wd, const T *dY, T *dX, float *dW, int accumulate,
                            Workspace &ws, hipStream_t s)
{
    const DenseConvPlan p = plan_dense_conv(g);
    const int npix = g.N * g.Ho * g.Wo, HW = g.Ho * g.Wo, kk = g.k * g.k;
    float *part = ws.take<float>(p.n_part);
    int st = PF_OK;
    if (g.N == 0) return accumulate ? st : launch_zero_f32(s, dW, (i64)g.Cout * g.C * kk);
    if (dX) {
        // the transposed convolution of the dense layer: the same gather with Cout in place of r
        st = launch_gemm_generic<T, true, false>("dense_conv_dX=Wt*dY", s,
                                                 GemmShape{g.C, g.N * g.H * g.W, g.Cout * kk, 1, 1},
                                                 OpA_FilterT<T>{Wd, g.C, kk}, OpB_Col2im<T>{dY, g, g.Cout},
                                                 EpiNCHW<T, T>{dX, nullptr, g.C, g.H * g.W});
        if (st != PF_OK) return st;
    }
    if (dW) {
        st = launch_gemm_generic<T, true, true>("dense_conv_dW=dY*Xcolt", s, GemmShape{g.Cout, g.C * kk, npix, 1, p.ks},
                                                OpA_NCHW<T>{dY, g.Cout, HW}, OpB_Im2colT<T>{OpB_Im2col<T>{X, g}},
                                                EpiPartial{part, (i64)g.C * kk, (i64)g.Cout * g.C * kk});
        if (st == PF_OK) st = launch_splitk_reduce(s, part, dW, (i64)g.Cout * g.C * kk, p.ks, accumulate);
    }
    return st;
}

} // namespace pf

using namespace pf;

extern "C" {

size_t pf_lowrank_conv_fwd_workspace_bytes(const pf_conv_desc *d)
{
    ConvGeom g;
    if (check_conv_desc(d, &g) != PF_OK) return 0;
    return plan_conv(g, d->dtype).fwd_bytes;
}

size_t pf_lowrank_conv_bwd_workspace_bytes(const pf_conv_desc *d)
{
    ConvGeom g;
    if (check_conv_desc(d, &g) != PF_OK) return 0;
    return plan_conv(g, d->dtype).bwd_bytes;
}

size_t pf_lowrank_conv_saved_weights_bytes(const pf_conv_desc *d)
{
    ConvGeom g;
    if (check_conv_desc(d, &g) != PF_OK) return 0;
    return d->dtype == PF_BF16 ? plan_conv(g, d->dtype).saved_bytes : 0;
}

int pf_lowrank_conv_fwd(const pf_conv_desc *d, const void *X, const void *Uk, const void *Vp, void *Y, void *T_save,
                        void *W_save, void *workspace, size_t workspace_bytes, void *stream)
{
    bool fused = false;
    return pf::conv_fwd_entry_ep(d, X, Uk, Vp, nullptr, nullptr, nullptr, PF_ACT_NONE, Y, T_save, W_save, workspace,
                                 workspace_bytes, stream, &fused);
}

int pf_lowrank_conv_bwd(const pf_conv_desc *d, const void *X, const void *Uk, const void *Vp, const void *dY,
                        const void *T_saved, const void *W_saved, void *dX, void *dUk, void *dVp, int accumulate,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    bool fused = false;
    return pf::conv_bwd_entry_ep(d, X, Uk, Vp, nullptr, dY, T_saved, W_saved, nullptr, 0, dX, dUk, dVp, accumulate,
                                 workspace, workspace_bytes, stream, &fused);
}

size_t pf_dense_conv_workspace_bytes(const pf_conv_desc *d)
{
    ConvGeom g;
    if (check_conv_desc(d, &g) != PF_OK) return 0;
    return plan_dense_conv(g).bytes;
}

int pf_dense_conv_fwd(const pf_conv_desc *d, const void *X, const void *Wd, void *Y, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    (void)workspace;
    (void)workspace_bytes;
    ConvGeom g;
    int st = check_conv_desc(d, &g);
    if (st != PF_OK) return st;
    if (!Wd) return PF_ERR_NULL;
    if (g.N == 0) return PF_OK;
    if (!X || !Y) return PF_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32) return dense_conv_fwd_t<float>(g, (const float *)X, (const float *)Wd, (float *)Y, s);
    return dense_conv_fwd_t<bf16_t>(g, (const bf16_t *)X, (const bf16_t *)Wd, (bf16_t *)Y, s);
}

int pf_dense_conv_bwd(const pf_conv_desc *d, const void *X, const void *Wd, const void *dY, void *dX, void *dWd,
                      int accumulate, void *workspace, size_t workspace_bytes, void *stream)
{
    ConvGeom g;
    int st = check_conv_desc(d, &g);
    if (st != PF_OK) return st;
    if (!Wd) return PF_ERR_NULL;
    if (g.N > 0 && (!X || !dY)) return PF_ERR_NULL;
    const size_t need = plan_dense_conv(g).bytes;
    if (!workspace || workspace_bytes < need) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32)
        return dense_conv_bwd_t<float>(g, (const float *)X, (const float *)Wd, (const float *)dY, (float *)dX,
                                       (float *)dWd, accumulate, ws, s);
    return dense_conv_bwd_t<bf16_t>(g, (const bf16_t *)X, (const bf16_t *)Wd, (const bf16_t *)dY, (bf16_t *)dX,
                                    (float *)dWd, accumulate, ws, s);
}

} // extern "C"

// Does the backward call for this descriptor run on the chain kernels, which fold a batch-norm scale into their
// weight re-ordering and into the sum of the filter gradients?  (Otherwise the caller scales beforehand.)
bool pf::conv_bwd_takes_scale(const pf_conv_desc *d, bool want_dX)
{
    ConvGeom g;
    if (check_conv_desc(d, &g) != PF_OK || d->dtype != PF_BF16 || g.N == 0 || !want_dX) return false;
    const ConvPlan p = plan_conv(g, d->dtype);
    return p.chain && p.wgrad;
}

// ------------------------------------------------ entry points with an epilogue
// (the element-wise part is applied by the caller when *fused stays false)
int pf::conv_fwd_entry_ep(const pf_conv_desc *d, const void *X, const void *Uk, const void *Vp, const float *scale,
                          const float *shift, const void *residual, int act, void *Y, void *T_save, void *W_save,
                          void *workspace, size_t workspace_bytes, void *stream, bool *fused)
{
    ConvGeom g;
    int st = check_conv_desc(d, &g);
    if (st != PF_OK) return st;
    if (!Uk || !Vp) return PF_ERR_NULL;
    if (g.N > 0 && (!X || !Y)) return PF_ERR_NULL;
    if (any_misaligned({X, Uk, Vp, Y, T_save, W_save}, 16)) return PF_ERR_UNSUPPORTED;
    const ConvPlan p = plan_conv(g, d->dtype);
    if (p.fwd_bytes > 0 && (!workspace || workspace_bytes < p.fwd_bytes)) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    if (g.N == 0) return PF_OK;
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    if (d->dtype == PF_F32)
        return conv_fwd_generic<float>(g, (const float *)X, (const float *)Uk, (const float *)Vp, (float *)Y,
                                       (float *)T_save, ws, s);
    if (p.chain)
    {
        // the kernel applies the epilogue as it stores (its float4 loads of scale and shift need 16-byte alignment)
        ConvEpilogue ep = {};
        if (!any_misaligned({scale, shift}, 16)) {
            ep = ConvEpilogue{scale, shift, residual, nullptr, act == PF_ACT_RELU ? 1 : 0};
            *fused = true;
        }
        return conv_fwd_chain(g, p, (const bf16_t *)X, (const bf16_t *)Uk, (const bf16_t *)Vp, (bf16_t *)Y,
                              (bf16_t *)T_save, W_save, ws, s, ep);
    }
    return conv_fwd_generic<bf16_t>(g, (const bf16_t *)X, (const bf16_t *)Uk, (const bf16_t *)Vp, (bf16_t *)Y,
                                    (bf16_t *)T_save, ws, s);
}

int pf::conv_bwd_entry_ep(const pf_conv_desc *d, const void *X, const void *Uk, const void *Vp, const float *scale,
                          const void *dY, const void *T_saved, const void *W_saved, const void *dX_add, int x_is_relu,
                          void *dX, void *dUk, void *dVp, int accumulate, void *workspace, size_t workspace_bytes,
                          void *stream, bool *fused)
{
    ConvGeom g;
    int st = check_conv_desc(d, &g);
    if (st != PF_OK) return st;
    if (!Uk || !Vp) return PF_ERR_NULL;
    if (g.N > 0 && (!X || !dY)) return PF_ERR_NULL;
    if (any_misaligned({X, Uk, Vp, dY, T_saved, W_saved, dX}, 16) || any_misaligned({dUk, dVp}, 4)) return PF_ERR_UNSUPPORTED;
    const ConvPlan p = plan_conv(g, d->dtype);
    if (p.bwd_bytes > 0 && (!workspace || workspace_bytes < p.bwd_bytes)) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    if (g.N == 0) {
        if (!accumulate) {
            st = launch_zero_f32(s, (float *)dUk, (i64)g.r * g.C * g.k * g.k);
            if (st == PF_OK) st = launch_zero_f32(s, (float *)dVp, (i64)g.Cout * g.r);
        }
        return st;
    }
    if (d->dtype == PF_F32)
        return conv_bwd_generic<float>(g, p, (const float *)X, (const float *)Uk, (const float *)Vp, (const float *)dY,
                                       (const float *)T_saved, (float *)dX, (float *)dUk, (float *)dVp, accumulate, ws,
                                       s);
    if (p.chain && dX)
    {
        *fused = true; // the kernel adds the skip gradient and masks as it stores dX
        return conv_bwd_chain(g, p, (const bf16_t *)X, (const bf16_t *)Uk, (const bf16_t *)Vp, (const bf16_t *)dY,
                              (const bf16_t *)T_saved, p.saved_bytes ? W_saved : nullptr, (bf16_t *)dX, (float *)dUk,
                              (float *)dVp, accumulate, ws, s, ConvEpilogue{scale, nullptr, dX_add, x_is_relu ? X : nullptr, 0});
    }
    return conv_bwd_generic<bf16_t>(g, p, (const bf16_t *)X, (const bf16_t *)Uk, (const bf16_t *)Vp,
                                    (const bf16_t *)dY, (const bf16_t *)T_saved, (bf16_t *)dX, (float *)dUk,
                                    (float *)dVp, accumulate, ws, s);
}
