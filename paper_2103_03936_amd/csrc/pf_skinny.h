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
constexpr int SK_MAX_PROB = 8;

struct SkinnyProb {
    const float *A; // activations, A[m * lda + k]
    const float *W; // weights, KN: W[k * ldw + n], NK: W[n * ldw + k]
    float *P;       // slice sums, P[ks * pcount + m * ldp + n]; only n < N is written
    i64 lda, ldw, pcount;
    int K, N, ldp;
    int ntiles, ksplit, kper, wg0; // filled by skinny_plan
};
struct SkinnyArgs {
    SkinnyProb p[SK_MAX_PROB];
    int nprob, M, nwg;
};
// Chooses the slicing of every problem (about `target` workgroups in all) and numbers the workgroups.
void skinny_plan(SkinnyArgs &a, int target = 256);
// Slices skinny_plan would pick for a contraction of length K among `total_tiles` column tiles.
int skinny_ksplit(i64 K, i64 total_tiles, int target = 256);
inline i64 skinny_tiles(i64 N) { return (N + SK_TILE_N - 1) / SK_TILE_N; }
int launch_skinny_gemm(hipStream_t s, const char *name, const SkinnyArgs &a, bool nk);

// out[m * ldo + n] = sum over ks < ksplit of P[ks * pcount + m * ldp + n], several segments in one launch
struct SliceSumSeg {
    const float *P;
    float *out;
    i64 pcount, ldo;
    int ldp, ksplit, N;
};
struct SliceSumArgs {
    SliceSumSeg s[4];
    int nseg, M;
};
int launch_slice_sum(hipStream_t s, const SliceSumArgs &a);

// out[i * ldo + j] (+)= sum_b A[b * lda + i] * Bm[b * ldb + j], b < M: the weight gradients of a cell are
// rank-M updates.  Bm == NULL stands for a column of ones (a bias gradient, J = 1).
struct RankProb {
    const float *A, *Bm;
    float *out;
    i64 lda, ldb, ldo;
    int I, J, wg0, jt; // jt = column tiles
};
constexpr int RK_MAX_PROB = 12;
struct RankArgs {
    RankProb p[RK_MAX_PROB];
    int nprob, M, accumulate, nwg;
};
void rank_add(RankArgs &a, const float *A, i64 lda, const float *Bm, i64 ldb, float *out, i64 ldo, int I, int J);
// seg: optional slice sums done by extra workgroups of the same launch (nseg == 0: none)
int launch_rank_update(hipStream_t s, const RankArgs &a, const SliceSumArgs &seg);

} // namespace pf
