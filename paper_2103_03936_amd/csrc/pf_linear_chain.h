// Fully connected low-rank layer as one kernel (bf16 in, fp32 accumulate), both factors read in place:
//     mid[rows][R] = in[rows][C1] * W1[C1][R],   out[rows][C2] = mid * W2[C2][R]^T (+ bias)
//   forward  (Section 2.1): in = X,  W1 = V,  W2 = U, mid = T  (kept on chip, copied out once for backward)
//   backward data:          in = dY, W1 = U,  W2 = V, mid = dT
// A workgroup owns 32 rows.  The contraction of stage 1 runs over the rows of W1, the slow index of a
// row-major factor, so W1 passes through LDS as it is and the MFMA fragments come out of it with the
// transposing LDS read; W2 is already contraction-fast and goes from global memory straight to registers.
#pragma once

#include "pf_common.h"

namespace pf {

struct LinChainArgs {
    const uint16_t *in;   // [rows][C1] bf16
    const uint16_t *W1;   // [C1][R] bf16
    const uint16_t *W2;   // [C2][R] bf16
    const uint16_t *bias; // [C2] bf16, nullable
    uint16_t *out;        // [rows][C2] bf16
    uint16_t *mid_save;   // [rows][R] bf16, nullable
    float *colsum;        // [2 * row tiles][C1] column sums of `in` per 16 rows, nullable
    i64 rows;
    int C1, C2;
    // Several layers of the same shape in one launch (groups > 1; 0 or 1: a single layer).  Each pointer above
    // moves by its stride (in elements) from one group to the next; a stride of 0 shares the operand.  With
    // sum_out the groups write ONE output, the sum of their stage-2 products (no bias then): the backward-data
    // pass of projections that share their input.
    int groups, sum_out;
    i64 gs_in, gs_W1, gs_W2, gs_bias, gs_out, gs_mid, gs_colsum;
    // Epilogue applied as the output leaves (single layer only; every member nullable / zero):
    //   out = mask > 0 ? act(out + add) : 0
    const uint16_t *ep_add;  // [rows][C2] bf16: a residual input, or a gradient arriving over a skip connection
    const uint16_t *ep_mask; // [rows][C2] bf16: the output is zero where this is not positive
    int ep_relu;             // act = max(0, .)
};

constexpr int LC_ROWS = 32; // rows per workgroup

// R == 128, C1 and C2 multiples of 256
bool linear_chain2_supported(i64 n_in, i64 n_out, i64 r);
// groups > 1: at most LC_MAX_GROUPS; with sum_out also C2 <= 512 (the sums stay in registers)
constexpr int LC_MAX_GROUPS = 8;
bool linear_chain2_multi_supported(i64 n_in, i64 n_out, i64 r, int groups, bool sum_out);
int launch_linear_chain2(hipStream_t s, const char *name, const LinChainArgs &a);

} // namespace pf
