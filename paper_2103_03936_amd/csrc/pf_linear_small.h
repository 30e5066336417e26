// Small-batch fp32 factorized linear layer (see pf_linear_small.hip): argument blocks and launchers.
#pragma once

#include "pf_common.h"

namespace pf {

constexpr int LS_MAX_K = 128;  // rows M, and rank r, at most (the contraction length of the second launch's tiles)
constexpr int LS_MAX_PROB = 4; // products of one tile launch
constexpr int LS_MAX_SLICES = 8;

// launch 1: P[s][m][n] = sum over k in slice s of A[m * lda + k] W[k * ldw + n]; K a multiple of 32 S, N of 32
struct LsSliceArgs {
    const float *A, *W;
    float *P;
    i64 lda, ldw;
    int M, K, N, S;
};
int linear_small_slices(i64 K); // slices for a contraction of length K (a multiple of 32): 8, 4, 2 or 1
int launch_ls_slices(hipStream_t s, const char *name, const LsSliceArgs &a0, const LsSliceArgs &a1 = LsSliceArgs{});

enum { LS_MK = 0, LS_KM = 1 };
// an operand of a tile product: element (i, k) at p[i * ld + k] (LS_MK) or p[k * ld + i] (LS_KM), summed over
// `slices` copies `sstride` floats apart
struct LsOperand {
    const float *p;
    i64 ld, sstride;
    int layout, slices;
};
inline LsOperand ls_operand(const float *p, i64 ld, int layout, int slices = 1, i64 sstride = 0)
{
    return LsOperand{p, ld, sstride, layout, slices};
}
// C[m * ldc + n] (+)= sum_k A(m, k) B(k, n) + bias[n], m < M, n < N, k < K <= LS_MAX_K.  A_copy (nullable): the
// (summed) left operand written once as [M][K].  colsum (nullable): colsum[m] (+)= sum_k A(m, k).  C may be NULL
// when only those are wanted.
struct LsTileProb {
    LsOperand A, B;
    float *C, *A_copy, *colsum;
    const float *bias;
    i64 ldc;
    int M, N, K, accumulate, wg0;
};
struct LsTileArgs {
    LsTileProb p[LS_MAX_PROB];
    int nprob, nwg;
};
void ls_add(LsTileArgs &a, const LsOperand &A, const LsOperand &B, int M, int N, int K, float *C, i64 ldc,
            const float *bias, int accumulate, float *A_copy = nullptr, float *colsum = nullptr);
int launch_ls_tiles(hipStream_t s, const char *name, const LsTileArgs &a);

// fp32, 0 < M <= 128, r <= 128, in / out / r multiples of 32
bool linear_small_supported(i64 M, i64 n_in, i64 n_out, i64 r);

} // namespace pf
