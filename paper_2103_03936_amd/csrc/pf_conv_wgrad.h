// Filter-gradient kernel for small images (see pf_conv_wgrad.hip).
#pragma once

#include "pf_common.h"

namespace pf {

struct WgradArgs {
    const uint16_t *A; // [N][M][H*W] bf16
    const uint16_t *B; // [N][Nc][H*W] bf16
    float *partial;    // [groups][taps][M][Nc]
    int M, Nc, H, W, N_img, imgs_per_group, groups;
    i64 rows; // fully connected layer only: total rows of A and B (N_img = number of 64-row tiles)
};

struct WgradReduceArgs {
    const float *partial; // [groups][taps][M][Nc]
    float *out;           // out[m * s_m + n * s_n + tap * s_tap]; NULL = nothing to do
    int groups, taps, M, Nc;
    i64 s_m, s_n, s_tap;
    int accumulate;
    const float *nscale; // nullable: the sum of column n is multiplied by nscale[n] (a fixed batch-norm scale)
};

// out[c] (+)= sum over tiles of partial[tile][c]; cols a multiple of 32
struct ColsumTilesArgs {
    const float *partial;
    float *out;
    int tiles, cols, accumulate;
};

bool wgrad_supported(int M, int Nc, int H, int W, int k, int stride, int pad);
int wgrad_nchunk(int M, int k, int which); // B channels per workgroup; which = 1 / 2: first / second problem of a pair
// Both filter gradients in one launch: a1 = the k1 x k1 stage, a2 = the 1x1 stage (partial == NULL skips one).
int launch_conv_wgrad_pair(hipStream_t s, const WgradArgs &a1, int k1, const WgradArgs &a2);
// The fully connected layer: A[rows][M], B[rows][Nc] row-major; Out[m][n] = sum_rows A[row][m] B[row][n].
int launch_linear_wgrad_pair(hipStream_t s, const WgradArgs &a1, const WgradArgs &a2, int cols = 256);
// cs (nullable): a column-sum problem for extra blocks of the same launch
int launch_wgrad_reduce(hipStream_t s, const WgradReduceArgs &r0, const WgradReduceArgs &r1,
                        const ColsumTilesArgs *cs = nullptr);

} // namespace pf
