// Products with a handful of activation rows (M <= 32: an LSTM cell at batch 20) in fp32:
//     C[M][N] = A[M][K] * W        with W stored [K][N] ("KN", N fast) or [N][K] ("NK", K fast).
// Every weight is used once per call, so the kernels are built to stream the weights once, at full width,
// from as many compute units as there are: the contraction is cut into slices, one workgroup per
// (128-column tile, slice), and the slices are added afterwards in a fixed order.
#pragma once

#include "pf_common.h"

namespace pf {

constexpr int SK_MAX_ROWS = 32;  // activation rows one MFMA tile holds
constexpr int SK_TILE_N = 128;   // output columns per workgroup
constexpr int SK_MAX_PROB = 16;

struct SkinnyProb {
    const float *A; // activations, A[m * lda + k]
    const float *W; // weights, KN: W[k * ldw + n], NK: W[n * ldw + k]
    float *P;       // slice sums, P[ks * pcount + m * ldp + n]; only n < N is written
    i64 lda, ldw, pcount;
    int M, K, N, ldp;              // M <= 32 rows of A (and of P) belong to this problem
    int ntiles, ksplit, kper, wg0; // filled by skinny_plan
};
struct SkinnyArgs {
    SkinnyProb p[SK_MAX_PROB];
    int wg0[SK_MAX_PROB]; // first workgroup of every problem once more, side by side: one scalar load finds a
                          // workgroup's problem (filled by skinny_plan; INT_MAX-like past nprob)
    int nprob, nwg;
};
// Chooses the slicing of every problem (about `target` workgroups in all) and numbers the workgroups.
void skinny_plan(SkinnyArgs &a, int target = 256);
// Slices skinny_plan would pick for a contraction of length K among `total_tiles` column tiles.
int skinny_ksplit(i64 K, i64 total_tiles, int target = 256);
inline i64 skinny_tiles(i64 N) { return (N + SK_TILE_N - 1) / SK_TILE_N; }
int launch_skinny_gemm(hipStream_t s, const char *name, const SkinnyArgs &a, bool nk);

// Weights that many launches reuse (a layer's factors over the steps of a sequence) can be copied once into the
// order the kernel consumes them in: for column tile `tile` and the eight contraction indices 8 S .. 8 S + 7, the
// 16 bytes of lane l for column sub-tile e are the four values W(k = 8 S + 4 (l / 32) + 0..3, n = 128 tile + 32 e
// + l % 32) at float offset (((tile * ceil(K / 8) + S) * 4 + e) * 64 + l) * 4, zero past K and N.  A wavefront's
// load is then one aligned kilobyte.  With such a copy W of a problem points at it and ldw is not used.
inline size_t skinny_packed_floats(int K, int N) { return (size_t)skinny_tiles(N) * (size_t)((K + 7) / 8) * 1024; }
struct SkinnyPackItem {
    const float *src; // element (k, n) at src[k * sk + n * sn]
    float *dst;
    i64 sk, sn, item0; // item0: the first 16-byte item of this matrix among all of the launch
    int K, N;
};
constexpr int SK_MAX_PACK = 8;
struct SkinnyPackArgs {
    SkinnyPackItem m[SK_MAX_PACK];
    int n;
    i64 items;
};
void skinny_pack_add(SkinnyPackArgs &a, const float *src, i64 sk, i64 sn, int K, int N, float *dst);
int launch_skinny_pack(hipStream_t s, const SkinnyPackArgs &a);
int launch_skinny_gemm_packed(hipStream_t s, const char *name, const SkinnyArgs &a);

// out[m * ldo + n] = bias[n] + sum over ks < ksplit of P[ks * pcount + m * ldp + n], m < M; several segments in
// one launch (bias nullable)
struct SliceSumSeg {
    const float *P, *bias;
    float *out;
    i64 pcount, ldo;
    int M, ldp, ksplit, N;
};
struct SliceSumArgs {
    SliceSumSeg s[4];
    int nseg;
};
int launch_slice_sum(hipStream_t s, const SliceSumArgs &a, const char *name = "slice_sum");

// For kernels that add the slices up themselves: the sum over n slices of P[k * pcount + idx], in order, eight
// loads in flight at a time (slices past the end add zero).
__device__ __forceinline__ float slices_at(const float *P, int n, i64 pcount, i64 idx)
{
    float s = 0.f;
    for (int k0 = 0; k0 < n; k0 += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + u;
            const float x = P[(i64)(k < n ? k : 0) * pcount + idx];
            v[u] = k < n ? x : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    return s;
}

inline SkinnyProb skinny_prob(int M, const float *A, i64 lda, const float *W, i64 ldw, int K, int N, int ldp,
                              i64 pcount)
{
    SkinnyProb p = {};
    p.M = M;
    p.A = A;
    p.W = W;
    p.lda = lda;
    p.ldw = ldw;
    p.K = K;
    p.N = N;
    p.ldp = ldp;
    p.pcount = pcount;
    return p;
}

// the slice sums of problem p into out[m * ldo + n], n < N
inline SliceSumSeg slice_seg(const SkinnyProb &p, float *out, i64 ldo, int N)
{
    SliceSumSeg s;
    s.P = p.P;
    s.bias = nullptr;
    s.M = p.M;
    s.out = out;
    s.pcount = p.pcount;
    s.ldo = ldo;
    s.ldp = p.ldp;
    s.ksplit = p.ksplit;
    s.N = N;
    return s;
}

// Row blocks of up to 32 rows of one product C[M x N] = A[M x K] W become the problems of one launch
// (M <= 32 * SK_MAX_PROB).  Places the slice sums from `part` on (NULL: size only) and returns the floats they take.
inline size_t skinny_rows(int M, const float *A, i64 lda, const float *W, i64 ldw, int K, int N, float *part,
                          SkinnyArgs &a)
{
    a = SkinnyArgs{};
    const i64 pc = (i64)M * N;
    for (int m0 = 0; m0 < M; m0 += SK_MAX_ROWS)
        a.p[a.nprob++] = skinny_prob(M - m0 < SK_MAX_ROWS ? M - m0 : SK_MAX_ROWS, A ? A + (i64)m0 * lda : nullptr, lda,
                                     W, ldw, K, N, N, pc);
    skinny_plan(a);
    for (int q = 0; q < a.nprob; ++q) a.p[q].P = part ? part + (i64)SK_MAX_ROWS * q * N : nullptr;
    return (size_t)(a.p[0].ksplit * pc); // every block has the same K and N, hence the same slicing
}
// all row blocks of such a product summed in one segment: out[m * ldo + n] (+ bias[n])
inline SliceSumSeg skinny_rows_seg(const SkinnyArgs &a, int M, float *out, i64 ldo, const float *bias)
{
    SliceSumSeg sg = slice_seg(a.p[0], out, ldo, a.p[0].N);
    sg.M = M;
    sg.bias = bias;
    return sg;
}

// out[i * ldo + j] (+)= sum_b A[b * lda + i] * Bm[b * ldb + j], b < M: the weight gradients of a cell are
// rank-M updates.  Bm == NULL stands for a column of ones (a bias gradient, J = 1).
struct RankProb {
    const float *A, *Bm;
    float *out;
    i64 lda, ldb, ldo;
    int M, I, J, wg0, jt; // M = rows summed over; jt = column tiles
};
constexpr int RK_MAX_PROB = 12;
struct RankArgs {
    RankProb p[RK_MAX_PROB];
    int nprob, M, accumulate, nwg; // M: rows of a problem added without a count of its own
};
void rank_add(RankArgs &a, const float *A, i64 lda, const float *Bm, i64 ldb, float *out, i64 ldo, int I, int J,
              int M = -1);
// seg: optional slice sums done by extra workgroups of the same launch (nseg == 0: none)
int launch_rank_update(hipStream_t s, const char *name, const RankArgs &a, const SliceSumArgs &seg);

struct __attribute__((packed, aligned(4))) F4u {
    float v[4];
};

// four floats at a 4-byte aligned address
__device__ __forceinline__ f32x4_t ld4(const float *p)
{
    const F4u t = *(const F4u *)p;
    f32x4_t r = {t.v[0], t.v[1], t.v[2], t.v[3]};
    return r;
}
// the first n of four floats (n <= 0: none), zero elsewhere; only the first n are touched
__device__ __forceinline__ f32x4_t ld4n(const float *p, int n)
{
    if (n >= 4) return ld4(p);
    f32x4_t r = {0.f, 0.f, 0.f, 0.f};
    if (n > 0) r[0] = p[0];
    if (n > 1) r[1] = p[1];
    if (n > 2) r[2] = p[2];
    return r;
}

// out (+)= [A0; A]^T * Bm on the matrix unit, for sums over hundreds of rows (the weight gradients of a whole
// sequence): out[i * ldo + j] (+)= sum_{b < M0} A0[b * lda + i] * Bm[b * ldb + j]
//                                + sum_{M0 <= b < M} A[(b - M0) * lda + i] * Bm[b * ldb + j].
// The two-part left operand is the hidden state one step back: h0, then h_0 .. h_{T-2}.
// colsum (optional): colsum[i] (+)= sum_b A[b][i], a bias gradient.
struct RankMmaProb {
    const float *A0, *A, *Bm;
    float *out, *colsum;
    i64 lda, ldb, ldo;
    int M0, M, I, J, wg0, jt, ntile, nwg; // jt = column tiles; nwg = ntile rounded up to a multiple of eight
};
constexpr int RM_MAX_PROB = 12;
struct RankMmaArgs {
    RankMmaProb p[RM_MAX_PROB];
    int nprob, accumulate, nwg, xi; // nwg, xi (tile height / 64) and the problems' tile fields: set by the launch
};
// false: the kernel does not take this problem (a row shorter than four floats, too many problems); out == NULL: skipped
bool rank_mma_add(RankMmaArgs &a, const float *A0, int M0, const float *A, i64 lda, const float *Bm, i64 ldb,
                  float *out, i64 ldo, int I, int J, int M, float *colsum = nullptr);
int launch_rank_mma(hipStream_t s, const char *name, const RankMmaArgs &a);

} // namespace pf
