// A stack of factorized LSTM layers over a whole sequence (paper Section 2.3, eq. (2); the 2-layer language
// model of Appendix D), small batches, fp32.  Same arithmetic as running the layers one after the other, but
// scheduled as a wavefront: layer l at time t only needs layer l - 1 at time t and itself at time t - 1, so
// slot s = l + t of the forward pass handles every layer that has a step there in the SAME launches (backward:
// the mirror image).  A step of the recurrence is a chain of short, latency-bound launches; the wavefront makes
// that chain T + L - 1 slots long instead of T L.
//
// Per forward slot: one launch for all T = (h Vh | x Vx) products, one for their slice sums, one for all
// z = T U^T products, one for the gates of all active layers.  The input path of layer 0 does not depend on any
// recurrence and is computed for all time steps up front; the input path of a higher layer reads the layer
// below at the same time step and rides in the slot's launches.  All parameter gradients are formed once per
// layer over all T B rows after the backward wavefront.
#include <vector>

#include "pf_gemm.h"
#include "pf_skinny.h"
#include "pf_common.h"

namespace pf {

constexpr int ST_MAX_LAYERS = 4;

__device__ __forceinline__ float st_sigmoid(float z) { return 1.0f / (1.0f + expf(-z)); }

// ---- gates of all active layers of a slot (blockIdx.y = position in the list) ----
struct StackGatesFwd {
    const float *P[ST_MAX_LAYERS];     // pre-activation slices, [nslices][B x 4h]
    const float *bias[ST_MAX_LAYERS];  // nullable
    const float *zadd[ST_MAX_LAYERS];  // nullable: pre-activations computed up front (layer 0's input path)
    const float *c_prev[ST_MAX_LAYERS];
    float *h_out[ST_MAX_LAYERS], *c_out[ST_MAX_LAYERS], *gates[ST_MAX_LAYERS];
    int nslices[ST_MAX_LAYERS];
    int n, B, h;
};

__global__ __launch_bounds__(256) void lstm_stack_gates_fwd_kernel(StackGatesFwd a)
{
    const int q = blockIdx.y, h = a.h;
    const i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (i64)a.B * h) return;
    const int b = (int)(idx / h), j = (int)(idx % h);
    const i64 base = (i64)b * 4 * h + j, pcount = (i64)a.B * 4 * h;
    float z[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) z[g] = slices_at(a.P[q], a.nslices[q], pcount, base + (i64)g * h);
    if (a.bias[q]) {
#pragma unroll
        for (int g = 0; g < 4; ++g) z[g] += a.bias[q][j + (i64)g * h];
    }
    if (a.zadd[q]) {
#pragma unroll
        for (int g = 0; g < 4; ++g) z[g] += a.zadd[q][base + (i64)g * h];
    }
    const float ig = st_sigmoid(z[0]), fg = st_sigmoid(z[1]), gg = tanhf(z[2]), og = st_sigmoid(z[3]);
    const float c = fg * a.c_prev[q][idx] + ig * gg;
    float *gt = a.gates[q];
    gt[base] = ig;
    gt[base + h] = fg;
    gt[base + 2 * (i64)h] = gg;
    gt[base + 3 * (i64)h] = og;
    a.c_out[q][idx] = c;
    a.h_out[q][idx] = og * tanhf(c);
}

// dh_t of a layer = what arrives from above (a tensor, or slices of dTx V_x^T of the layer above) + what arrives
// from its own step t + 1 (a tensor for the last step, else slices of dTh V_h^T); then the gate derivatives.
struct StackGatesBwd {
    const float *gates[ST_MAX_LAYERS], *c_prev[ST_MAX_LAYERS], *c_out[ST_MAX_LAYERS];
    const float *dh_a[ST_MAX_LAYERS], *dh_b[ST_MAX_LAYERS];       // tensors [B x h], nullable
    const float *P1[ST_MAX_LAYERS], *P2[ST_MAX_LAYERS];           // slice sets [n][B x h], nullable when n == 0
    const float *dc_next[ST_MAX_LAYERS];                          // nullable
    float *dz[ST_MAX_LAYERS], *dc_prev[ST_MAX_LAYERS];
    int n1[ST_MAX_LAYERS], n2[ST_MAX_LAYERS];
    int n, B, h;
};

__global__ __launch_bounds__(256) void lstm_stack_gates_bwd_kernel(StackGatesBwd a)
{
    const int q = blockIdx.y, h = a.h;
    const i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (i64)a.B * h) return;
    const int b = (int)(idx / h), j = (int)(idx % h);
    const i64 base = (i64)b * 4 * h + j, pc = (i64)a.B * h;
    float dhv = (a.dh_a[q] ? a.dh_a[q][idx] : 0.f) + (a.dh_b[q] ? a.dh_b[q][idx] : 0.f);
    dhv += slices_at(a.P1[q], a.n1[q], pc, idx) + slices_at(a.P2[q], a.n2[q], pc, idx);
    const float *gt = a.gates[q];
    const float ig = gt[base], fg = gt[base + h], gg = gt[base + 2 * (i64)h], og = gt[base + 3 * (i64)h];
    const float tc = tanhf(a.c_out[q][idx]);
    const float dc = (a.dc_next[q] ? a.dc_next[q][idx] : 0.f) + dhv * og * (1.f - tc * tc);
    a.dc_prev[q][idx] = dc * fg;
    float *dz = a.dz[q];
    dz[base] = dc * gg * ig * (1.f - ig);
    dz[base + h] = dc * a.c_prev[q][idx] * fg * (1.f - fg);
    dz[base + 2 * (i64)h] = dc * ig * (1.f - gg * gg);
    dz[base + 3 * (i64)h] = dhv * tc * og * (1.f - og);
}

// ---- a launch (or a few) of skinny products whose slice sums are laid out region by region ----
// Problems of one region write different columns of the same slices (the four gate blocks of a z product), so
// they must get the same slicing: same K, same launch.
struct SkItem {
    SkinnyProb p;
    int region;
    i64 coloff;
};
struct SkBatch {
    std::vector<SkItem> items;
    std::vector<size_t> region_off, region_len; // floats, filled by run()
    std::vector<int> region_ksplit;
    int nregions = 0;
    int new_region() { return nregions++; }
    void add(const SkinnyProb &p, int region, i64 coloff = 0) { items.push_back(SkItem{p, region, coloff}); }
    // Plans every launch (at most SK_MAX_PROB problems each, regions kept whole), places the slices from `part`
    // on (NULL: sizes only; cap floats are there) and launches unless dry.  *used: the floats of `part` taken.
    int run(hipStream_t s, const char *name, bool nk, float *part, size_t cap, bool dry, size_t *used, bool packed = true)
    {
        region_off.assign(nregions, 0);
        region_len.assign(nregions, 0);
        region_ksplit.assign(nregions, 0);
        std::vector<SkinnyArgs> launches;
        size_t off = 0, i = 0;
        while (i < items.size()) {
            // the chunk: whole regions while they fit
            size_t j = i;
            while (j < items.size()) {
                size_t k = j;
                while (k < items.size() && items[k].region == items[j].region) ++k;
                if (k - i > (size_t)SK_MAX_PROB) break;
                j = k;
            }
            if (j == i) return PF_ERR_UNSUPPORTED; // a region larger than a launch
            SkinnyArgs a = {};
            for (size_t k = i; k < j; ++k) a.p[a.nprob++] = items[k].p;
            skinny_plan(a);
            for (size_t k = i; k < j; ++k) {
                const SkinnyProb &pl = a.p[k - i];
                const int r = items[k].region;
                const size_t len = (size_t)pl.ksplit * (size_t)pl.pcount;
                if (region_ksplit[r] == 0) {
                    region_ksplit[r] = pl.ksplit;
                    region_len[r] = len;
                    region_off[r] = off;
                    off += len;
                } else if (region_ksplit[r] != pl.ksplit || region_len[r] != len) {
                    return PF_ERR_UNSUPPORTED;
                }
                a.p[k - i].P = part ? part + region_off[r] + items[k].coloff : nullptr;
            }
            launches.push_back(a);
            i = j;
        }
        if (used) *used = off;
        if (dry) return PF_OK;
        if (!part || off > cap) return PF_ERR_WORKSPACE;
        int st = PF_OK;
        for (size_t q = 0; q < launches.size() && st == PF_OK; ++q)
            st = packed ? launch_skinny_gemm_packed(s, name, launches[q]) : launch_skinny_gemm(s, name, launches[q], nk);
        return st;
    }
};

struct StackGeom {
    int T, B, din, h, r, G, gr, L;
    bool has_bias;
};

static int check_stack_desc(const pf_lstm_stack_desc *d, StackGeom *g)
{
    if (!d) return PF_ERR_NULL;
    if (d->dtype != PF_F32) return PF_ERR_UNSUPPORTED;
    if (d->groups != 1 && d->groups != 4) return PF_ERR_UNSUPPORTED;
    if (d->T < 0 || d->B < 0 || d->d_in <= 0 || d->h <= 0 || d->r <= 0) return PF_ERR_SHAPE;
    if (d->layers < 1 || d->layers > ST_MAX_LAYERS) return PF_ERR_SHAPE;
    const i64 lim = 0x7fffffffLL;
    if (d->T > lim || d->B > lim || d->d_in > lim || d->h > lim / 4 || d->r > lim / 4) return PF_ERR_SHAPE;
    if (d->T * d->B > lim || d->T * d->B * d->h * 4 > (lim << 3) || d->T * d->B * d->d_in > (lim << 3)) return PF_ERR_SHAPE;
    // built on the few-row streaming products: B <= 32 and every extent at least 4
    if (d->T > 0 && d->B > 0 && (d->B > SK_MAX_ROWS || d->d_in < 4 || d->h < 4 || d->r < 4)) return PF_ERR_UNSUPPORTED;
    if (g)
        *g = StackGeom{(int)d->T, (int)d->B, (int)d->d_in, (int)d->h, (int)d->r, d->groups, (int)(d->groups * d->r),
                       d->layers, d->has_bias != 0};
    return PF_OK;
}

// C[Mt x N] = A[Mt x K] W (+ bias) for Mt = T B rows, 256 rows per launch pair (product + slice sums)
constexpr int ST_ROWS = SK_MAX_ROWS * SK_MAX_PROB;
static int st_tall(hipStream_t s, const char *name, bool nk, i64 Mt, const float *A, i64 lda, const float *W, i64 ldw,
                   int K, int N, float *out, i64 ldo, const float *bias, float *part)
{
    int st = PF_OK;
    for (i64 m0 = 0; m0 < Mt && st == PF_OK; m0 += ST_ROWS) {
        const int Mg = (int)(Mt - m0 < ST_ROWS ? Mt - m0 : ST_ROWS);
        SkinnyArgs a;
        skinny_rows(Mg, A + m0 * lda, lda, W, ldw, K, N, part, a);
        st = launch_skinny_gemm(s, name, a, nk);
        if (st != PF_OK) break;
        SliceSumArgs ss = {};
        ss.s[ss.nseg++] = skinny_rows_seg(a, Mg, out + m0 * ldo, ldo, bias);
        st = launch_slice_sum(s, ss);
    }
    return st;
}
static size_t st_tall_part(i64 Mt, int K, int N)
{
    SkinnyArgs a;
    size_t m = 0;
    const int full = (int)(Mt < ST_ROWS ? Mt : ST_ROWS), last = (int)(Mt % ST_ROWS);
    if (full > 0) m = skinny_rows(full, nullptr, K, nullptr, N, K, N, nullptr, a);
    if (last > 0) {
        const size_t v = skinny_rows(last, nullptr, K, nullptr, N, K, N, nullptr, a);
        if (v > m) m = v;
    }
    return m;
}

// slice sums of several regions, four segments per launch
static int st_slice_sums(hipStream_t s, const std::vector<SliceSumSeg> &segs, const char *name)
{
    int st = PF_OK;
    for (size_t i = 0; i < segs.size() && st == PF_OK; i += 4) {
        SliceSumArgs ss = {};
        for (size_t k = i; k < segs.size() && k < i + 4; ++k) ss.s[ss.nseg++] = segs[k];
        st = launch_slice_sum(s, ss, name);
    }
    return st;
}
static SliceSumSeg st_seg(const float *P, i64 pcount, int ldp, int ksplit, int M, int N, float *out, i64 ldo)
{
    SliceSumSeg sg;
    sg.P = P;
    sg.bias = nullptr;
    sg.out = out;
    sg.pcount = pcount;
    sg.ldo = ldo;
    sg.M = M;
    sg.ldp = ldp;
    sg.ksplit = ksplit;
    sg.N = N;
    return sg;
}

// Per-layer tensors of the two entry points (host arrays of device pointers, copied)
struct StackPtrs {
    const float *h0[ST_MAX_LAYERS], *c0[ST_MAX_LAYERS];
    const float *Vx[ST_MAX_LAYERS], *Ux[ST_MAX_LAYERS], *Vh[ST_MAX_LAYERS], *Uh[ST_MAX_LAYERS], *bias[ST_MAX_LAYERS];
    float *h_all[ST_MAX_LAYERS], *c_all[ST_MAX_LAYERS], *gates_all[ST_MAX_LAYERS], *Tx_all[ST_MAX_LAYERS],
        *Th_all[ST_MAX_LAYERS];
};

// The factors in the order the streaming kernel reads them (see skinny_packed_floats), copied once per call: every
// one of the T + L - 1 slots reuses them.  Forward roles: T = a V (contraction over V's rows), z = T U^T (over U's
// columns); backward roles: dT = dz U (over U's rows), dh = dT V^T (over V's columns).
struct StackPacked {
    const float *Vh[ST_MAX_LAYERS], *Vx[ST_MAX_LAYERS];       // Vx: layers above the first only
    const float *Uh[ST_MAX_LAYERS][4], *Ux[ST_MAX_LAYERS][4]; // per gate block when every gate has its own pair
};
// Places the copies from buf on (NULL: sizes only), launches the copy kernels unless dry; returns the floats taken.
static size_t stack_pack(const StackGeom &g, const StackPtrs &p, bool bwd, float *buf, StackPacked *out, bool dry,
                         hipStream_t s, int *status)
{
    const int h = g.h, r = g.r, gr = g.gr, nq = g.G == 1 ? 1 : 4;
    size_t off = 0;
    int st = PF_OK;
    SkinnyPackArgs pa = {};
    auto flush = [&]() {
        if (!dry && st == PF_OK && pa.n > 0) st = launch_skinny_pack(s, pa);
        pa = SkinnyPackArgs{};
    };
    auto add = [&](const float *src, i64 sk, i64 sn, int K, int N) -> const float * {
        float *dst = buf ? buf + off : nullptr;
        off += skinny_packed_floats(K, N);
        if (!dry) {
            skinny_pack_add(pa, src, sk, sn, K, N, dst);
            if (pa.n == SK_MAX_PACK) flush();
        }
        return dst;
    };
    for (int l = 0; l < g.L; ++l) {
        for (int path = 0; path < 2; ++path) { // 0: hidden path, 1: input path (hoisted for the first layer)
            if (path == 1 && l == 0) continue;
            const float *V = dry ? nullptr : (path ? p.Vx[l] : p.Vh[l]), *U = dry ? nullptr : (path ? p.Ux[l] : p.Uh[l]);
            // V is [h x gr]: forward contracts over its rows, backward over its columns
            const float *pv = bwd ? add(V, 1, gr, gr, h) : add(V, gr, 1, h, gr);
            if (out) (path ? out->Vx : out->Vh)[l] = pv;
            for (int q = 0; q < nq; ++q) {
                // U (or its gate block q) is [rows x r] with rows = 4h or h
                const int rows = g.G == 1 ? 4 * h : h;
                const float *Uq = U ? U + (i64)q * h * r : nullptr;
                const float *pu = bwd ? add(Uq, r, 1, rows, r) : add(Uq, 1, r, r, rows);
                if (out) (path ? out->Ux : out->Uh)[l][q] = pu;
            }
        }
    }
    flush();
    if (status) *status = st;
    return off;
}

// ---- forward slot: products and gates of the layers in `mask` (layer l at time t = slot - l) ----
// part (NULL: sizes only) holds the slices of one launch group at a time.
static int stack_fwd_slot(const StackGeom &g, const StackPtrs &p, const StackPacked &pk, const float *zx0, int slot,
                          float *part, size_t cap,
                          bool dry, hipStream_t s, size_t *need)
{
    const int B = g.B, h = g.h, r = g.r, G = g.G, gr = g.gr;
    const i64 Bh = (i64)B * h;
    int st = PF_OK;
    size_t used = 0, most = 0;
    // T = h_{t-1} Vh, and for layers above the first T = x_t Vx with x_t = the layer below at time t
    SkBatch kn;
    int reg_th[ST_MAX_LAYERS], reg_tx[ST_MAX_LAYERS];
    for (int l = 0; l < g.L; ++l) {
        const int t = slot - l;
        reg_th[l] = reg_tx[l] = -1;
        if (t < 0 || t >= g.T) continue;
        const float *hp = dry ? nullptr : (t ? p.h_all[l] + (i64)(t - 1) * Bh : p.h0[l]);
        reg_th[l] = kn.new_region();
        kn.add(skinny_prob(B, hp, h, pk.Vh[l], gr, h, gr, gr, (i64)B * gr), reg_th[l]);
        if (l > 0) {
            reg_tx[l] = kn.new_region();
            kn.add(skinny_prob(B, dry ? nullptr : p.h_all[l - 1] + (i64)t * Bh, h, pk.Vx[l], gr, h, gr, gr, (i64)B * gr),
                   reg_tx[l]);
        }
    }
    st = kn.run(s, "lstm_stack_T", false, part, cap, dry, &used);
    if (st != PF_OK) return st;
    most = used;
    if (!dry) {
        std::vector<SliceSumSeg> segs;
        for (int l = 0; l < g.L; ++l) {
            const int t = slot - l;
            if (reg_th[l] >= 0)
                segs.push_back(st_seg(part + kn.region_off[reg_th[l]], (i64)B * gr, gr, kn.region_ksplit[reg_th[l]], B, gr,
                                      p.Th_all[l] + (i64)t * B * gr, gr));
            if (reg_tx[l] >= 0)
                segs.push_back(st_seg(part + kn.region_off[reg_tx[l]], (i64)B * gr, gr, kn.region_ksplit[reg_tx[l]], B, gr,
                                      p.Tx_all[l] + (i64)t * B * gr, gr));
        }
        st = st_slice_sums(s, segs, "lstm_stack_T_sum");
        if (st != PF_OK) return st;
    }
    // z slices = Th Uh^T (and Tx Ux^T above the first layer), one region per product, a layer's regions adjacent
    SkBatch nk;
    int reg_zh[ST_MAX_LAYERS], reg_zx[ST_MAX_LAYERS];
    const i64 pcz = (i64)B * 4 * h;
    auto add_z = [&](int region, const float *Tm, const float *const *U) { // U: the packed gate blocks
        if (G == 1) {
            nk.add(skinny_prob(B, Tm, gr, U[0], r, r, 4 * h, 4 * h, pcz), region);
        } else {
            for (int q = 0; q < 4; ++q)
                nk.add(skinny_prob(B, Tm ? Tm + (i64)q * r : nullptr, gr, U[q], r, r, h, 4 * h, pcz), region, (i64)q * h);
        }
    };
    for (int l = 0; l < g.L; ++l) {
        const int t = slot - l;
        reg_zh[l] = reg_zx[l] = -1;
        if (t < 0 || t >= g.T) continue;
        reg_zh[l] = nk.new_region();
        add_z(reg_zh[l], dry ? nullptr : p.Th_all[l] + (i64)t * B * gr, pk.Uh[l]);
        if (l > 0) {
            reg_zx[l] = nk.new_region();
            add_z(reg_zx[l], dry ? nullptr : p.Tx_all[l] + (i64)t * B * gr, pk.Ux[l]);
        }
    }
    st = nk.run(s, "lstm_stack_z", true, part, cap, dry, &used);
    if (st != PF_OK) return st;
    if (used > most) most = used;
    if (need) *need = most;
    if (dry) return st;
    StackGatesFwd ga = {};
    ga.B = B;
    ga.h = h;
    for (int l = 0; l < g.L; ++l) {
        const int t = slot - l;
        if (t < 0 || t >= g.T) continue;
        const int q = ga.n++;
        ga.P[q] = part + nk.region_off[reg_zh[l]];
        ga.nslices[q] = nk.region_ksplit[reg_zh[l]] + (l > 0 ? nk.region_ksplit[reg_zx[l]] : 0);
        // (a layer's two regions were created one after the other, so their slices are adjacent)
        ga.bias[q] = (l > 0 && g.has_bias) ? p.bias[l] : nullptr; // layer 0's bias is inside zx0
        ga.zadd[q] = l == 0 ? zx0 + (i64)t * pcz : nullptr;
        ga.c_prev[q] = t ? p.c_all[l] + (i64)(t - 1) * Bh : p.c0[l];
        ga.h_out[q] = p.h_all[l] + (i64)t * Bh;
        ga.c_out[q] = p.c_all[l] + (i64)t * Bh;
        ga.gates[q] = p.gates_all[l] + (i64)t * pcz;
    }
    const dim3 grid((unsigned)((Bh + 255) / 256), (unsigned)ga.n);
    PF_LAUNCH(st, "lstm_stack_gates_fwd", lstm_stack_gates_fwd_kernel, grid, dim3(256), s, ga);
    return st;
}

struct StackPlan {
    size_t n_zx0, n_part, n_part2, n_dT, n_dz, n_pack_f, n_pack_b, fwd_bytes, bwd_bytes;
};

// per-layer tensors of the backward pass
struct StackBwdPtrs {
    const float *dhT[ST_MAX_LAYERS], *dcT[ST_MAX_LAYERS];
    float *dh0[ST_MAX_LAYERS], *dc0[ST_MAX_LAYERS];
    float *dVx[ST_MAX_LAYERS], *dUx[ST_MAX_LAYERS], *dVh[ST_MAX_LAYERS], *dUh[ST_MAX_LAYERS], *dbias[ST_MAX_LAYERS];
    float *dz_all[ST_MAX_LAYERS], *dTh_all[ST_MAX_LAYERS], *dTx_all[ST_MAX_LAYERS]; // workspace
};

// ---- backward slot u: layer l at time t with (L - 1 - l) + (T - 1 - t) = u ----
// part: slices of the dT products (consumed by the slice sums of the same slot); part2: slices of dh_{t-1} and of
// the dx handed to the layer below, consumed by the gate kernel of the NEXT slot, whose layout `prev` records.
struct StackCarry {
    const float *P1[ST_MAX_LAYERS], *P2[ST_MAX_LAYERS]; // for layer l: recurrent slices / slices from layer l + 1
    int n1[ST_MAX_LAYERS], n2[ST_MAX_LAYERS];
};
static int stack_bwd_slot(const StackGeom &g, const StackPtrs &p, const StackPacked &pk, const StackBwdPtrs &b,
                          const float *dh_top, int u,
                          float *part, size_t cap, float *part2, size_t cap2, StackCarry &carry, bool dry, hipStream_t s,
                          size_t *need, size_t *need2)
{
    const int B = g.B, h = g.h, r = g.r, G = g.G, gr = g.gr, L = g.L, T = g.T;
    const i64 Bh = (i64)B * h, pcz = (i64)B * 4 * h;
    int st = PF_OK;
    auto time_of = [&](int l) { return T - 1 - (u - (L - 1 - l)); };
    auto active = [&](int l) {
        const int t = time_of(l);
        return t >= 0 && t < T;
    };
    if (!dry) {
        StackGatesBwd ga = {};
        ga.B = B;
        ga.h = h;
        for (int l = 0; l < L; ++l) {
            if (!active(l)) continue;
            const int t = time_of(l), q = ga.n++;
            ga.gates[q] = p.gates_all[l] + (i64)t * pcz;
            ga.c_prev[q] = t ? p.c_all[l] + (i64)(t - 1) * Bh : p.c0[l];
            ga.c_out[q] = p.c_all[l] + (i64)t * Bh;
            ga.dh_a[q] = l == L - 1 ? dh_top + (i64)t * Bh : nullptr; // the top layer's dL/dh_t comes from outside
            ga.dh_b[q] = t == T - 1 ? b.dhT[l] : nullptr;
            ga.P1[q] = carry.P1[l];
            ga.n1[q] = t == T - 1 ? 0 : carry.n1[l];
            ga.P2[q] = carry.P2[l];
            ga.n2[q] = l == L - 1 ? 0 : carry.n2[l];
            // dc_t lives in dc0 between the steps of a layer (each element is read, then rewritten, by its own thread)
            ga.dc_next[q] = t == T - 1 ? b.dcT[l] : b.dc0[l];
            ga.dz[q] = b.dz_all[l] + (i64)t * pcz;
            ga.dc_prev[q] = b.dc0[l];
        }
        const dim3 grid((unsigned)((Bh + 255) / 256), (unsigned)ga.n);
        PF_LAUNCH(st, "lstm_stack_gates_bwd", lstm_stack_gates_bwd_kernel, grid, dim3(256), s, ga);
        if (st != PF_OK) return st;
    }
    // dTh = dz Uh, and above the first layer dTx = dz Ux (layer 0's input path is done for all steps at the end)
    SkBatch kn;
    int reg_h[ST_MAX_LAYERS], reg_x[ST_MAX_LAYERS];
    const i64 pcT = (i64)B * gr;
    auto add_dT = [&](int region, const float *dz, const float *const *U) { // U: the packed gate blocks
        if (G == 1) {
            kn.add(skinny_prob(B, dz, 4 * (i64)h, U[0], r, 4 * h, r, gr, pcT), region);
        } else {
            for (int q = 0; q < 4; ++q)
                kn.add(skinny_prob(B, dz ? dz + (i64)q * h : nullptr, 4 * (i64)h, U[q], r, h, r, gr, pcT), region,
                       (i64)q * r);
        }
    };
    for (int l = 0; l < L; ++l) {
        reg_h[l] = reg_x[l] = -1;
        if (!active(l)) continue;
        const int t = time_of(l);
        const float *dz = dry ? nullptr : b.dz_all[l] + (i64)t * pcz;
        reg_h[l] = kn.new_region();
        add_dT(reg_h[l], dz, pk.Uh[l]);
        if (l > 0) {
            reg_x[l] = kn.new_region();
            add_dT(reg_x[l], dz, pk.Ux[l]);
        }
    }
    size_t used = 0;
    st = kn.run(s, "lstm_stack_dT", false, part, cap, dry, &used);
    if (st != PF_OK) return st;
    if (need) *need = used;
    if (!dry) {
        std::vector<SliceSumSeg> segs;
        for (int l = 0; l < L; ++l) {
            if (!active(l)) continue;
            const int t = time_of(l);
            segs.push_back(st_seg(part + kn.region_off[reg_h[l]], pcT, gr, kn.region_ksplit[reg_h[l]], B, gr,
                                  b.dTh_all[l] + (i64)t * pcT, gr));
            if (l > 0)
                segs.push_back(st_seg(part + kn.region_off[reg_x[l]], pcT, gr, kn.region_ksplit[reg_x[l]], B, gr,
                                      b.dTx_all[l] + (i64)t * pcT, gr));
        }
        st = st_slice_sums(s, segs, "lstm_stack_dT_sum");
        if (st != PF_OK) return st;
    }
    // slices of dh_{t-1} = dTh Vh^T for the layer itself and of dx_t = dTx Vx^T for the layer below
    SkBatch nk;
    int reg_dh[ST_MAX_LAYERS], reg_dx[ST_MAX_LAYERS];
    for (int l = 0; l < L; ++l) {
        reg_dh[l] = reg_dx[l] = -1;
        if (!active(l)) continue;
        const int t = time_of(l);
        reg_dh[l] = nk.new_region();
        nk.add(skinny_prob(B, dry ? nullptr : b.dTh_all[l] + (i64)t * pcT, gr, pk.Vh[l], gr, gr, h, h, Bh),
               reg_dh[l]);
        if (l > 0) {
            reg_dx[l] = nk.new_region();
            nk.add(skinny_prob(B, dry ? nullptr : b.dTx_all[l] + (i64)t * pcT, gr, pk.Vx[l], gr, gr, h, h, Bh),
                   reg_dx[l]);
        }
    }
    st = nk.run(s, "lstm_stack_dh", true, part2, cap2, dry, &used);
    if (st != PF_OK) return st;
    if (need2) *need2 = used;
    if (dry) return st;
    std::vector<SliceSumSeg> last;
    for (int l = 0; l < L; ++l) {
        if (!active(l)) continue;
        carry.P1[l] = part2 + nk.region_off[reg_dh[l]];
        carry.n1[l] = nk.region_ksplit[reg_dh[l]];
        if (l > 0) {
            carry.P2[l - 1] = part2 + nk.region_off[reg_dx[l]];
            carry.n2[l - 1] = nk.region_ksplit[reg_dx[l]];
        }
        if (time_of(l) == 0) // the gradient that reaches the layer's initial state
            last.push_back(st_seg(carry.P1[l], Bh, h, carry.n1[l], B, h, b.dh0[l], h));
    }
    return st_slice_sums(s, last, "lstm_stack_dh0_sum");
}

static int plan_stack(const StackGeom &g, StackPlan *out)
{
    StackPlan p = {};
    const i64 Mt = (i64)g.T * g.B;
    if (Mt == 0) {
        *out = p;
        return PF_OK;
    }
    p.n_zx0 = (size_t)(Mt * 4 * g.h);
    p.n_dz = p.n_zx0;
    p.n_dT = (size_t)(Mt * g.gr);
    size_t m = 0, m2 = 0;
    auto upd = [&](size_t v) {
        if (v > m) m = v;
    };
    upd(st_tall_part(Mt, g.din, g.gr));                    // Tx = X Vx, layer 0
    upd(st_tall_part(Mt, g.r, g.G == 1 ? 4 * g.h : g.h));  // zx = Tx Ux^T
    upd(st_tall_part(Mt, g.G == 1 ? 4 * g.h : g.h, g.r));  // dTx = dz Ux
    upd(st_tall_part(Mt, g.gr, g.din));                    // dx = dTx Vx^T
    StackPtrs none = {};
    StackPacked nonep = {};
    StackBwdPtrs noneb = {};
    StackCarry carry = {};
    for (int slot = 0; slot < g.T + g.L - 1; ++slot) {
        // the sets of active layers repeat: every slot in the middle has all of them
        if (slot >= g.L && slot < g.T - 1) continue;
        size_t need = 0, need2 = 0;
        int st = stack_fwd_slot(g, none, nonep, nullptr, slot, nullptr, 0, true, nullptr, &need);
        if (st != PF_OK) return st;
        upd(need);
        st = stack_bwd_slot(g, none, nonep, noneb, nullptr, slot, nullptr, 0, nullptr, 0, carry, true, nullptr, &need, &need2);
        if (st != PF_OK) return st;
        upd(need);
        if (need2 > m2) m2 = need2;
    }
    p.n_part = m;
    p.n_part2 = m2;
    p.n_pack_f = stack_pack(g, none, false, nullptr, nullptr, true, nullptr, nullptr);
    p.n_pack_b = stack_pack(g, none, true, nullptr, nullptr, true, nullptr, nullptr);
    p.fwd_bytes = align_up(p.n_zx0 * sizeof(float)) + align_up(p.n_part * sizeof(float)) + align_up(p.n_pack_f * sizeof(float));
    p.bwd_bytes = (size_t)g.L * (align_up(p.n_dz * sizeof(float)) + 2 * align_up(p.n_dT * sizeof(float))) +
                  align_up(p.n_part * sizeof(float)) + align_up(p.n_part2 * sizeof(float)) +
                  align_up(p.n_pack_b * sizeof(float));
    *out = p;
    return PF_OK;
}

} // namespace pf

using namespace pf;

extern "C" {

size_t pf_lowrank_lstm_stack_fwd_workspace_bytes(const pf_lstm_stack_desc *d)
{
    StackGeom g;
    StackPlan p;
    if (check_stack_desc(d, &g) != PF_OK || plan_stack(g, &p) != PF_OK) return 0;
    return p.fwd_bytes;
}

size_t pf_lowrank_lstm_stack_bwd_workspace_bytes(const pf_lstm_stack_desc *d)
{
    StackGeom g;
    StackPlan p;
    if (check_stack_desc(d, &g) != PF_OK || plan_stack(g, &p) != PF_OK) return 0;
    return p.bwd_bytes;
}

int pf_lowrank_lstm_stack_fwd(const pf_lstm_stack_desc *d, const void *x, const void *const *h0, const void *const *c0,
                              const void *const *Vx, const void *const *Ux, const void *const *Vh,
                              const void *const *Uh, const void *const *bias, void *const *h_all, void *const *c_all,
                              void *const *gates_all, void *const *Tx_all, void *const *Th_all, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    StackGeom g;
    int st = check_stack_desc(d, &g);
    if (st != PF_OK) return st;
    if (!h0 || !c0 || !Vx || !Ux || !Vh || !Uh || (g.has_bias && !bias) || !h_all || !c_all || !gates_all || !Tx_all ||
        !Th_all)
        return PF_ERR_NULL;
    StackPtrs p = {};
    for (int l = 0; l < g.L; ++l) {
        if (!Vx[l] || !Ux[l] || !Vh[l] || !Uh[l] || (g.has_bias && !bias[l])) return PF_ERR_NULL;
        if (g.T > 0 && g.B > 0 && (!h0[l] || !c0[l] || !h_all[l] || !c_all[l] || !gates_all[l] || !Tx_all[l] || !Th_all[l]))
            return PF_ERR_NULL;
        if (any_misaligned({h0[l], c0[l], Vx[l], Ux[l], Vh[l], Uh[l], g.has_bias ? bias[l] : nullptr, h_all[l], c_all[l],
                            gates_all[l], Tx_all[l], Th_all[l]},
                           16))
            return PF_ERR_UNSUPPORTED;
        p.h0[l] = (const float *)h0[l];
        p.c0[l] = (const float *)c0[l];
        p.Vx[l] = (const float *)Vx[l];
        p.Ux[l] = (const float *)Ux[l];
        p.Vh[l] = (const float *)Vh[l];
        p.Uh[l] = (const float *)Uh[l];
        p.bias[l] = g.has_bias ? (const float *)bias[l] : nullptr;
        p.h_all[l] = (float *)h_all[l];
        p.c_all[l] = (float *)c_all[l];
        p.gates_all[l] = (float *)gates_all[l];
        p.Tx_all[l] = (float *)Tx_all[l];
        p.Th_all[l] = (float *)Th_all[l];
    }
    if (g.T == 0 || g.B == 0) return PF_OK;
    if (!x || any_misaligned({x}, 16)) return x ? PF_ERR_UNSUPPORTED : PF_ERR_NULL;
    StackPlan pl;
    st = plan_stack(g, &pl);
    if (st != PF_OK) return st;
    if (!workspace || workspace_bytes < pl.fwd_bytes) return PF_ERR_WORKSPACE;
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    float *zx0 = ws.take<float>(pl.n_zx0);
    float *part = ws.take<float>(pl.n_part);
    float *packed = ws.take<float>(pl.n_pack_f);
    StackPacked pk = {};
    stack_pack(g, p, false, packed, &pk, false, s, &st);
    if (st != PF_OK) return st;
    const i64 Mt = (i64)g.T * g.B;
    const int h = g.h, r = g.r, gr = g.gr;
    // the input path of the first layer for every time step at once
    st = st_tall(s, "lstm_stack_Tx0=X*Vx", false, Mt, (const float *)x, g.din, p.Vx[0], gr, g.din, gr, p.Tx_all[0], gr,
                 nullptr, part);
    if (st != PF_OK) return st;
    if (g.G == 1) {
        st = st_tall(s, "lstm_stack_zx0=Tx*Uxt", true, Mt, p.Tx_all[0], gr, p.Ux[0], r, r, 4 * h, zx0, 4 * (i64)h,
                     p.bias[0], part);
    } else {
        for (int q = 0; q < 4 && st == PF_OK; ++q)
            st = st_tall(s, "lstm_stack_zx0=Tx*Uxt", true, Mt, p.Tx_all[0] + (i64)q * r, gr, p.Ux[0] + (i64)q * h * r, r, r,
                         h, zx0 + (i64)q * h, 4 * (i64)h, p.bias[0] ? p.bias[0] + (i64)q * h : nullptr, part);
    }
    for (int slot = 0; slot < g.T + g.L - 1 && st == PF_OK; ++slot)
        st = stack_fwd_slot(g, p, pk, zx0, slot, part, pl.n_part, false, s, nullptr);
    return st;
}

int pf_lowrank_lstm_stack_bwd(const pf_lstm_stack_desc *d, const void *x, const void *const *h0, const void *const *c0,
                              const void *const *h_all, const void *const *c_all, const void *const *gates_all,
                              const void *const *Tx_all, const void *const *Th_all, const void *const *Vx,
                              const void *const *Ux, const void *const *Vh, const void *const *Uh, const void *dh_top,
                              const void *const *dhT, const void *const *dcT, void *dx_all, void *const *dh0,
                              void *const *dc0, void *const *dVx, void *const *dUx, void *const *dVh, void *const *dUh,
                              void *const *dbias, int accumulate, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    StackGeom g;
    int st = check_stack_desc(d, &g);
    if (st != PF_OK) return st;
    if (!h0 || !c0 || !h_all || !c_all || !gates_all || !Tx_all || !Th_all || !Vx || !Ux || !Vh || !Uh || !dh0 || !dc0 ||
        !dVx || !dUx || !dVh || !dUh)
        return PF_ERR_NULL;
    StackPtrs p = {};
    StackBwdPtrs b = {};
    hipStream_t s = (hipStream_t)stream;
    const int L = g.L, h = g.h, r = g.r, gr = g.gr, B = g.B, T = g.T;
    for (int l = 0; l < L; ++l) {
        if (!Vx[l] || !Ux[l] || !Vh[l] || !Uh[l] || !dVx[l] || !dUx[l] || !dVh[l] || !dUh[l]) return PF_ERR_NULL;
        if (T > 0 && B > 0 &&
            (!h0[l] || !c0[l] || !h_all[l] || !c_all[l] || !gates_all[l] || !Tx_all[l] || !Th_all[l] || !dh0[l] || !dc0[l]))
            return PF_ERR_NULL;
        if (any_misaligned({h0[l], c0[l], h_all[l], c_all[l], gates_all[l], Tx_all[l], Th_all[l], Vx[l], Ux[l], Vh[l], Uh[l],
                            dhT ? dhT[l] : nullptr, dcT ? dcT[l] : nullptr, dh0[l], dc0[l]},
                           16) ||
            any_misaligned({dVx[l], dUx[l], dVh[l], dUh[l], dbias ? dbias[l] : nullptr}, 4))
            return PF_ERR_UNSUPPORTED;
        p.h0[l] = (const float *)h0[l];
        p.c0[l] = (const float *)c0[l];
        p.h_all[l] = (float *)h_all[l];
        p.c_all[l] = (float *)c_all[l];
        p.gates_all[l] = (float *)gates_all[l];
        p.Tx_all[l] = (float *)Tx_all[l];
        p.Th_all[l] = (float *)Th_all[l];
        p.Vx[l] = (const float *)Vx[l];
        p.Ux[l] = (const float *)Ux[l];
        p.Vh[l] = (const float *)Vh[l];
        p.Uh[l] = (const float *)Uh[l];
        b.dhT[l] = dhT ? (const float *)dhT[l] : nullptr;
        b.dcT[l] = dcT ? (const float *)dcT[l] : nullptr;
        b.dh0[l] = (float *)dh0[l];
        b.dc0[l] = (float *)dc0[l];
        b.dVx[l] = (float *)dVx[l];
        b.dUx[l] = (float *)dUx[l];
        b.dVh[l] = (float *)dVh[l];
        b.dUh[l] = (float *)dUh[l];
        b.dbias[l] = dbias ? (float *)dbias[l] : nullptr;
    }
    if (T == 0 || B == 0) { // no rows: the gradients this call owns are zero
        for (int l = 0; l < L && st == PF_OK && !accumulate; ++l) {
            const i64 din = l ? h : g.din;
            st = launch_zero_f32(s, b.dVx[l], din * gr);
            if (st == PF_OK) st = launch_zero_f32(s, b.dVh[l], (i64)h * gr);
            if (st == PF_OK) st = launch_zero_f32(s, b.dUx[l], 4 * (i64)h * r);
            if (st == PF_OK) st = launch_zero_f32(s, b.dUh[l], 4 * (i64)h * r);
            if (st == PF_OK) st = launch_zero_f32(s, b.dbias[l], 4 * (i64)h);
        }
        return st;
    }
    if (!x || !dh_top) return PF_ERR_NULL;
    if (any_misaligned({x, dh_top, dx_all}, 16)) return PF_ERR_UNSUPPORTED;
    StackPlan pl;
    st = plan_stack(g, &pl);
    if (st != PF_OK) return st;
    if (!workspace || workspace_bytes < pl.bwd_bytes) return PF_ERR_WORKSPACE;
    Workspace ws(workspace, workspace_bytes);
    for (int l = 0; l < L; ++l) {
        b.dz_all[l] = ws.take<float>(pl.n_dz);
        b.dTh_all[l] = ws.take<float>(pl.n_dT);
        b.dTx_all[l] = ws.take<float>(pl.n_dT);
    }
    float *part = ws.take<float>(pl.n_part);
    float *part2 = ws.take<float>(pl.n_part2);
    float *packed = ws.take<float>(pl.n_pack_b);
    StackPacked pk = {};
    stack_pack(g, p, true, packed, &pk, false, s, &st);
    if (st != PF_OK) return st;
    StackCarry carry = {};
    for (int u = 0; u < T + L - 1 && st == PF_OK; ++u)
        st = stack_bwd_slot(g, p, pk, b, (const float *)dh_top, u, part, pl.n_part, part2, pl.n_part2, carry, false, s,
                            nullptr, nullptr);
    if (st != PF_OK) return st;
    // the input path of the first layer for all steps at once
    const i64 Mt = (i64)T * B;
    if (g.G == 1) {
        st = st_tall(s, "lstm_stack_dTx0=dz*Ux", false, Mt, b.dz_all[0], 4 * (i64)h, p.Ux[0], r, 4 * h, r, b.dTx_all[0], gr,
                     nullptr, part);
    } else {
        for (int q = 0; q < 4 && st == PF_OK; ++q)
            st = st_tall(s, "lstm_stack_dTx0=dz*Ux", false, Mt, b.dz_all[0] + (i64)q * h, 4 * (i64)h,
                         p.Ux[0] + (i64)q * h * r, r, h, r, b.dTx_all[0] + (i64)q * r, gr, nullptr, part);
    }
    if (st != PF_OK) return st;
    if (dx_all) {
        st = st_tall(s, "lstm_stack_dx=dTx*Vxt", true, Mt, b.dTx_all[0], gr, p.Vx[0], gr, gr, g.din, (float *)dx_all, g.din,
                     nullptr, part);
        if (st != PF_OK) return st;
    }
    // parameter gradients, layer by layer, each a few rank-(T B) updates in one launch
    const SliceSumArgs none = {};
    for (int l = 0; l < L && st == PF_OK; ++l) {
        const float *xin = l ? p.h_all[l - 1] : (const float *)x;
        const int din = l ? h : g.din;
        RankArgs ra = {};
        ra.M = (int)Mt;
        ra.accumulate = accumulate;
        for (int path = 0; path < 2; ++path) {
            const float *Tm = path ? p.Th_all[l] : p.Tx_all[l];
            float *dU = path ? b.dUh[l] : b.dUx[l];
            if (g.G == 1) {
                rank_add(ra, b.dz_all[l], 4 * (i64)h, Tm, gr, dU, r, 4 * h, r);
            } else {
                for (int q = 0; q < 4; ++q)
                    rank_add(ra, b.dz_all[l] + (i64)q * h, 4 * (i64)h, Tm + (i64)q * r, gr, dU + (i64)q * h * r, r, h, r);
            }
        }
        rank_add(ra, xin, din, b.dTx_all[l], gr, b.dVx[l], gr, din, gr);
        // dVh = sum_t h_{t-1}^T dTh_t: the rows t >= 1 here, the h0 row block in a second launch below
        if (T > 1) rank_add(ra, p.h_all[l], h, b.dTh_all[l] + (i64)B * gr, gr, b.dVh[l], gr, h, gr, (int)(Mt - B));
        if (b.dbias[l]) rank_add(ra, b.dz_all[l], 4 * (i64)h, nullptr, 0, b.dbias[l], 1, 4 * h, 1);
        st = launch_rank_update(s, "lstm_stack_grads", ra, none);
        if (st != PF_OK) return st;
        RankArgs rb = {};
        rb.M = B;
        rb.accumulate = (T > 1) ? 1 : accumulate;
        rank_add(rb, p.h0[l], h, b.dTh_all[l], gr, b.dVh[l], gr, h, gr);
        st = launch_rank_update(s, "lstm_stack_grads", rb, none);
    }
    return st;
}

} // extern "C"
