// fp32 products with at most 32 activation rows (see pf_skinny.h), the slice sums, and rank-M updates.
//
// Operand layout of the 32x32x2 fp32 MFMA: lane l supplies A(row l % 32, k = l / 32) and
// B(k = l / 32, column l % 32); accumulator element v of lane l is C(8 (v / 4) + 4 (l / 32) + v % 4, l % 32).
// Activations are the A operand (rows past M read as zero), weights the B operand.  One "super-step"
// covers 8 consecutive k: lane l holds k = k0 + 4 (l / 32) + 0..3 as one 16-byte load, and the s-th of four
// MFMAs takes element s from both halves of the wavefront, i.e. k0 + s and k0 + 4 + s.
//   KN weights: 16 bytes = 4 neighbouring columns of one k -> the four column tiles of a wavefront are the
//               interleaved column sets n0 + 4 (l % 32) + j, j = 0..3; one load per k (4 per super-step).
//   NK weights: 16 bytes = 4 neighbouring k of one column -> column tiles n0 + 32 j + l % 32; one load per tile.
// Either way a super-step is 5 loads and 16 MFMAs for 128 columns.
#include "pf_skinny.h"

namespace pf {

// MODE 0: KN weights, 1: NK weights, 2: weights copied into the kernel's own order by skinny_pack_kernel
template <int MODE>
__global__ __launch_bounds__(256, 1) void skinny_gemm_kernel(SkinnyArgs a)
{
    constexpr bool NK = MODE != 0; // the packed order keeps NK's assignment of columns to lanes
    constexpr bool PK = MODE == 2;
    // partial tiles of the four wavefronts, two column tiles at a time
    __shared__ float red[4][2][16][64];

    int pi = 0;
#pragma unroll
    for (int q = 1; q < SK_MAX_PROB; ++q)
        if ((int)blockIdx.x >= a.wg0[q]) pi = q;
    const SkinnyProb &pb = a.p[pi];
    const float *__restrict__ A = pb.A;
    const float *__restrict__ W = pb.W;
    const i64 lda = pb.lda, ldw = pb.ldw;
    const int K = pb.K, N = pb.N, M = pb.M;
    const int local = blockIdx.x - pb.wg0, tile = local % pb.ntiles, ks = local / pb.ntiles;
    const int n0 = tile * SK_TILE_N;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, i = lane & 31;

    // this wavefront's contiguous quarter of the slice
    const int kw = pb.kper / 4;
    const int kA = ks * pb.kper + w * kw;
    const int kB = min(K, kA + kw);

    const bool row_ok = i < M;
    const float *Ap = A + (row_ok ? i : 0) * lda;

    // Every load is unconditional.  Addresses that would leave the matrix are pulled back inside it
    // (K >= 4 and N >= 4): a k that is pulled back is cancelled by zeroing the activation that multiplies
    // it, a column that is pulled back only recomputes a neighbour and is not stored twice differently.
    const int nbase = min(n0 + 4 * i, N - 4); // KN: this lane's four columns are nbase + j
    i64 nrow[4];                              // NK: this lane's column of tile j
#pragma unroll
    for (int j = 0; j < 4; ++j) nrow[j] = (i64)min(n0 + 32 * j + i, N - 1) * ldw;

    struct Stage { // one chunk = 4 super-steps = 32 k
        f32x4_t act[4];
        f32x4_t wv[4][4];
    };
    auto load_chunk = [&](Stage &st, int c) __attribute__((always_inline)) {
        if (kA + 32 * c >= kB) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int kk = kA + 32 * c + 8 * q + 4 * half; // this lane's k values: kk .. kk + 3
            const int kc = min(kk, K - 4);                 // where they are read from
            st.act[q] = ld4(Ap + kc); // masked when it is used
            if (!NK) {
#pragma unroll
                for (int e = 0; e < 4; ++e) st.wv[q][e] = ld4(W + (i64)(kc + e) * ldw + nbase);
            }
        }
        if (PK) {
            const i64 S_total = (K + 7) / 8;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const i64 S = min((i64)((kA + 32 * c + 8 * q) >> 3), S_total - 1); // past K: loaded, never used
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    st.wv[q][e] = *(const f32x4_t *)(W + ((((i64)tile * S_total + S) * 4 + e) * 64 + lane) * 4);
            }
        }
        // NK: a lane's loads of one column are neighbours in memory (32 k = one 128-byte stretch per chunk); issued
        // back to back they meet in the cache instead of fetching the line once per super-step
        if (NK && !PK) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int kc = min(kA + 32 * c + 8 * q + 4 * half, K - 4);
                    st.wv[q][e] = ld4(W + nrow[e] + kc);
                }
        }
    };

    f32x16_t tot[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) tot[j][v] = 0.f;

    // A fresh accumulator per 32-deep chunk, added to the running total: keeps the rounding error of a long
    // contraction at the level of its pairwise sum.
    auto compute_chunk = [&](const Stage &st, int c) __attribute__((always_inline)) {
        if (kA + 32 * c >= kB) return;
        f32x16_t cur[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) cur[j][v] = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (kA + 32 * c + 8 * q < kB) { // uniform
                const int kk = kA + 32 * c + 8 * q + 4 * half, kc = min(kk, K - 4);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    // KN / NK: weights and activations were read from kc, so element s stands for k = kc + s.
                    // Packed weights sit at their own k = kk + s: the activation is taken from where that k landed.
                    float av;
                    if (PK) {
                        const int idx = kk - kc + s;
                        const float pick = idx == 0 ? st.act[q][0] : idx == 1 ? st.act[q][1] : idx == 2 ? st.act[q][2] : st.act[q][3];
                        av = (row_ok && kk + s < kB) ? pick : 0.f;
                    } else {
                        av = (row_ok && kc + s >= kk && kc + s < kB) ? st.act[q][s] : 0.f;
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        cur[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, NK ? st.wv[q][j][s] : st.wv[q][s][j], cur[j], 0,
                                                                      0, 0);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) tot[j] += cur[j];
    };

    const int nch = kB > kA ? (kB - kA + 31) / 32 : 0;
    Stage s0, s1;
    load_chunk(s0, 0);
    load_chunk(s1, 1);
    for (int c = 0; c < nch; c += 2) {
        compute_chunk(s0, c);
        load_chunk(s0, c + 2);
        compute_chunk(s1, c + 1);
        load_chunk(s1, c + 3);
    }

    // add the four wavefronts' tiles in a fixed order and store the slice sum
    float *P = pb.P + (i64)ks * pb.pcount;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if (pass) __syncthreads();
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[w][t][v][lane] = tot[2 * pass + t][v];
        __syncthreads();
        const int t = w >> 1, j = 2 * pass + t;
#pragma unroll
        for (int vv = 0; vv < 8; ++vv) {
            const int v = 8 * (w & 1) + vv;
            const float sum = (red[0][t][v][lane] + red[1][t][v][lane]) + (red[2][t][v][lane] + red[3][t][v][lane]);
            const int m = 8 * (v >> 2) + 4 * half + (v & 3);
            const int n = NK ? n0 + 32 * j + i : nbase + j;
            if (m < M && (NK ? n : n0 + 4 * i) < N) P[(i64)m * pb.ldp + n] = sum;
        }
    }
}

int skinny_ksplit(i64 K, i64 total_tiles, int target)
{
    i64 want = total_tiles > 0 ? target / total_tiles : 1;
    if (want < 1) want = 1;
    i64 kper = ((K + want - 1) / want + 31) / 32 * 32;
    if (kper < 32) kper = 32;
    return (int)((K + kper - 1) / kper);
}

void skinny_plan(SkinnyArgs &a, int target)
{
    i64 total = 0;
    for (int q = 0; q < a.nprob; ++q) total += skinny_tiles(a.p[q].N);
    int wg = 0;
    for (int q = 0; q < a.nprob; ++q) {
        SkinnyProb &p = a.p[q];
        p.ntiles = (int)skinny_tiles(p.N);
        p.ksplit = skinny_ksplit(p.K, total, target);
        p.kper = (int)(((p.K + p.ksplit - 1) / p.ksplit + 31) / 32 * 32);
        p.wg0 = wg;
        wg += p.ntiles * p.ksplit;
    }
    for (int q = 0; q < SK_MAX_PROB; ++q) a.wg0[q] = q < a.nprob ? a.p[q].wg0 : 0x7fffffff;
    a.nwg = wg;
}

int launch_skinny_gemm(hipStream_t s, const char *name, const SkinnyArgs &a, bool nk)
{
    int st = PF_OK;
    if (a.nwg <= 0 || a.nprob <= 0) return st;
    if (a.nprob > SK_MAX_PROB) return PF_ERR_UNSUPPORTED;
    // the kernel pulls 16-byte loads back inside the matrix by up to three elements: both extents must hold four
    for (int q = 0; q < a.nprob; ++q)
        if (a.p[q].M < 1 || a.p[q].M > SK_MAX_ROWS || a.p[q].K < 4 || a.p[q].N < 4 || a.p[q].lda < a.p[q].K ||
            a.p[q].ldw < (nk ? a.p[q].K : a.p[q].N))
            return PF_ERR_UNSUPPORTED;
    if (nk) {
        PF_LAUNCH(st, name, skinny_gemm_kernel<1>, dim3(a.nwg), dim3(256), s, a);
    } else {
        PF_LAUNCH(st, name, skinny_gemm_kernel<0>, dim3(a.nwg), dim3(256), s, a);
    }
    return st;
}

int launch_skinny_gemm_packed(hipStream_t s, const char *name, const SkinnyArgs &a)
{
    int st = PF_OK;
    if (a.nwg <= 0 || a.nprob <= 0) return st;
    if (a.nprob > SK_MAX_PROB) return PF_ERR_UNSUPPORTED;
    for (int q = 0; q < a.nprob; ++q)
        if (a.p[q].M < 1 || a.p[q].M > SK_MAX_ROWS || a.p[q].K < 4 || a.p[q].N < 4 || a.p[q].lda < a.p[q].K ||
            ((uintptr_t)a.p[q].W & 15))
            return PF_ERR_UNSUPPORTED;
    PF_LAUNCH(st, name, skinny_gemm_kernel<2>, dim3(a.nwg), dim3(256), s, a);
    return st;
}

// one thread per 16-byte item of the packed order
__global__ __launch_bounds__(256) void skinny_pack_kernel(SkinnyPackArgs a)
{
    const i64 g = (i64)blockIdx.x * 256 + threadIdx.x;
    if (g >= a.items) return;
    int pi = 0;
#pragma unroll
    for (int q = 1; q < SK_MAX_PACK; ++q)
        if (q < a.n && g >= a.m[q].item0) pi = q;
    const SkinnyPackItem &m = a.m[pi];
    const i64 it = g - m.item0, S_total = (m.K + 7) / 8;
    const int lane = (int)(it & 63), e = (int)((it >> 6) & 3);
    const i64 S = (it >> 8) % S_total, tile = (it >> 8) / S_total;
    const i64 n = tile * SK_TILE_N + 32 * e + (lane & 31);
    f32x4_t v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const i64 k = 8 * S + 4 * (lane >> 5) + s;
        if (k < m.K && n < m.N) v[s] = m.src[k * m.sk + n * m.sn];
    }
    *(f32x4_t *)(m.dst + it * 4) = v;
}

void skinny_pack_add(SkinnyPackArgs &a, const float *src, i64 sk, i64 sn, int K, int N, float *dst)
{
    if (a.n >= SK_MAX_PACK) return;
    SkinnyPackItem &m = a.m[a.n++];
    m.src = src;
    m.dst = dst;
    m.sk = sk;
    m.sn = sn;
    m.K = K;
    m.N = N;
    m.item0 = a.items;
    a.items += (i64)(skinny_packed_floats(K, N) / 4);
}

int launch_skinny_pack(hipStream_t s, const SkinnyPackArgs &a)
{
    int st = PF_OK;
    if (a.n <= 0 || a.items <= 0) return st;
    for (int q = 0; q < a.n; ++q)
        if (!a.m[q].src || !a.m[q].dst || ((uintptr_t)a.m[q].dst & 15)) return PF_ERR_UNSUPPORTED;
    PF_LAUNCH(st, "skinny_pack", skinny_pack_kernel, dim3((unsigned)((a.items + 255) / 256)), dim3(256), s, a);
    return st;
}

// ------------------------------------------------------------------ slice sums
// A block takes 64 outputs at a time; four threads share an output, each adds every fourth slice (eight loads in
// flight), and the four sums are added in a fixed order.  `sh` is 256 floats of LDS.
__device__ __forceinline__ void slice_sum_block(const SliceSumArgs &a, int block, int nblocks, float *sh)
{
    const int e = threadIdx.x & 63, sg = threadIdx.x >> 6;
    for (int q = 0; q < a.nseg; ++q) {
        const SliceSumSeg &sg_ = a.s[q];
        const i64 count = (i64)sg_.M * sg_.N;
        for (i64 base = (i64)block * 64; base < count; base += (i64)nblocks * 64) { // uniform trip count
            const i64 idx = base + e;
            const bool ok = idx < count;
            const int m = (int)((ok ? idx : 0) / sg_.N), n = (int)((ok ? idx : 0) % sg_.N);
            const float *p = sg_.P + (i64)m * sg_.ldp + n;
            float acc = 0.f;
            int ks = sg;
            for (; ks + 28 < sg_.ksplit; ks += 32) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = p[(i64)(ks + 4 * u) * sg_.pcount];
#pragma unroll
                for (int u = 0; u < 8; ++u) acc += v[u];
            }
            { // the last round, again with every load in flight before the first add (slices past the end add zero)
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int k = ks + 4 * u;
                    const float x = p[(i64)(k < sg_.ksplit ? k : 0) * sg_.pcount];
                    v[u] = k < sg_.ksplit ? x : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) acc += v[u];
            }
            __syncthreads();
            sh[threadIdx.x] = acc;
            __syncthreads();
            if (sg == 0 && ok)
                sg_.out[(i64)m * sg_.ldo + n] =
                    ((sh[e] + sh[64 + e]) + (sh[128 + e] + sh[192 + e])) + (sg_.bias ? sg_.bias[n] : 0.f);
        }
    }
}

__global__ __launch_bounds__(256) void slice_sum_kernel(SliceSumArgs a)
{
    __shared__ float sh[256];
    slice_sum_block(a, blockIdx.x, gridDim.x, sh);
}

static int slice_sum_blocks(const SliceSumArgs &a)
{
    i64 most = 0;
    for (int q = 0; q < a.nseg; ++q) {
        const i64 c = (i64)a.s[q].M * a.s[q].N;
        if (c > most) most = c;
    }
    i64 nb = (most + 63) / 64;
    if (nb > 2048) nb = 2048;
    return (int)nb;
}

int launch_slice_sum(hipStream_t s, const SliceSumArgs &a, const char *name)
{
    int st = PF_OK;
    const int nb = slice_sum_blocks(a);
    if (nb <= 0) return st;
    PF_LAUNCH(st, name, slice_sum_kernel, dim3(nb), dim3(256), s, a);
    return st;
}

// ------------------------------------------------------------------ rank-M updates
constexpr int RK_TI = 32, RK_TJ = 128;

__global__ __launch_bounds__(256) void rank_update_kernel(RankArgs a, SliceSumArgs seg, int nseg_blocks)
{
    __shared__ __attribute__((aligned(16))) float As[SK_MAX_ROWS][RK_TI];
    __shared__ __attribute__((aligned(16))) float Bs[SK_MAX_ROWS][RK_TJ];
    if ((int)blockIdx.x >= a.nwg) { // the extra workgroups do the slice sums
        slice_sum_block(seg, blockIdx.x - a.nwg, nseg_blocks, &Bs[0][0]);
        return;
    }
    int pi = 0;
#pragma unroll
    for (int q = 1; q < RK_MAX_PROB; ++q)
        if (q < a.nprob && (int)blockIdx.x >= a.p[q].wg0) pi = q;
    const RankProb &pb = a.p[pi];
    const int local = blockIdx.x - pb.wg0;
    const int i0 = (local / pb.jt) * RK_TI, j0 = (local % pb.jt) * RK_TJ;
    const int tid = threadIdx.x, ti = tid >> 5, tj = tid & 31;
    const int I = pb.I, J = pb.J;

    float acc[4][4];
    // start from the old values when accumulating: their loads overlap the staging below
    const bool vec = j0 + 4 * tj + 4 <= J;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int ii = i0 + 4 * ti + e;
        const float *o = pb.out + (i64)(ii < I ? ii : 0) * pb.ldo + j0 + 4 * tj;
        f32x4_t old = {0.f, 0.f, 0.f, 0.f};
        if (a.accumulate && ii < I) old = vec ? ld4(o) : ld4n(o, J - (j0 + 4 * tj));
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[e][f] = old[f];
    }

    for (int b0 = 0; b0 < pb.M; b0 += SK_MAX_ROWS) {
        const int nb = min(SK_MAX_ROWS, pb.M - b0);
        if (b0) __syncthreads();
        // 16-byte pieces, all of a thread's requests in flight together (rows are only 4-byte aligned)
        if (tid < nb * (RK_TI / 4)) {
            const int b = tid / (RK_TI / 4), i4 = 4 * (tid % (RK_TI / 4));
            const int left = I - (i0 + i4);
            *(f32x4_t *)&As[b][i4] = ld4n(pb.A + (i64)(b0 + b) * pb.lda + (left > 0 ? i0 + i4 : 0), left);
        }
        f32x4_t bv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + 256 * q, b = e / (RK_TJ / 4), j4 = 4 * (e % (RK_TJ / 4));
            const int left = J - (j0 + j4);
            bv[q] = f32x4_t{1.f, 1.f, 1.f, 1.f};
            if (e < nb * (RK_TJ / 4) && pb.Bm) bv[q] = ld4n(pb.Bm + (i64)(b0 + b) * pb.ldb + (left > 0 ? j0 + j4 : 0), left);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + 256 * q, b = e / (RK_TJ / 4), j4 = 4 * (e % (RK_TJ / 4));
            const int left = J - (j0 + j4);
            if (e < nb * (RK_TJ / 4)) {
                f32x4_t v = bv[q];
#pragma unroll
                for (int f = 0; f < 4; ++f) v[f] = f < left ? v[f] : 0.f; // past J: zero (also for the ones column)
                *(f32x4_t *)&Bs[b][j4] = v;
            }
        }
        __syncthreads();
        for (int b = 0; b < nb; ++b) {
            const f32x4_t av = *(const f32x4_t *)&As[b][4 * ti];
            const f32x4_t bv = *(const f32x4_t *)&Bs[b][4 * tj];
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int f = 0; f < 4; ++f) acc[e][f] += av[e] * bv[f];
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int ii = i0 + 4 * ti + e;
        if (ii >= I) continue;
        float *o = pb.out + (i64)ii * pb.ldo + j0 + 4 * tj;
        if (vec) {
            F4u t;
#pragma unroll
            for (int f = 0; f < 4; ++f) t.v[f] = acc[e][f];
            *(F4u *)o = t;
        } else {
#pragma unroll
            for (int f = 0; f < 4; ++f)
                if (j0 + 4 * tj + f < J) o[f] = acc[e][f];
        }
    }
}

void rank_add(RankArgs &a, const float *A, i64 lda, const float *Bm, i64 ldb, float *out, i64 ldo, int I, int J, int M)
{
    if (!out || a.nprob >= RK_MAX_PROB) return;
    RankProb &p = a.p[a.nprob];
    p.A = A;
    p.Bm = Bm;
    p.out = out;
    p.lda = lda;
    p.ldb = ldb;
    p.ldo = ldo;
    p.M = M >= 0 ? M : a.M;
    p.I = I;
    p.J = J;
    p.jt = (J + RK_TJ - 1) / RK_TJ;
    p.wg0 = a.nwg;
    a.nwg += ((I + RK_TI - 1) / RK_TI) * p.jt;
    ++a.nprob;
}

int launch_rank_update(hipStream_t s, const char *name, const RankArgs &a, const SliceSumArgs &seg)
{
    int st = PF_OK;
    const int nsb = seg.nseg > 0 ? slice_sum_blocks(seg) : 0;
    if (a.nwg + nsb <= 0) return st;
    PF_LAUNCH(st, name, rank_update_kernel, dim3(a.nwg + nsb), dim3(256), s, a, seg, nsb);
    return st;
}

} // namespace pf
