// Fused two-stage convolution chain for small images (bf16 in, fp32 accumulate):
//     in[n][C1][HW] --(K1 x K1 conv, C1 -> R)--> mid[n][R][HW] --(K2 x K2 conv, R -> C2)--> out[n][C2][HW]
// with "same" geometry (stride 1; pad 1 for 3x3, pad 0 for 1x1) and H*W <= 64, so one
// workgroup owns one whole image and the rank-R intermediate never leaves the chip
// (it is optionally copied out once for the backward pass).
//   forward  (Section 2.2): in = X,  stage 1 = thin k x k filters Uk, stage 2 = 1x1 filters Vp,  mid = T
//   backward data:          in = dY, stage 1 = Vp^T (1x1),           stage 2 = flipped Uk (k x k), mid = dT
//
// Work split inside a workgroup (4 wavefronts):
//   stage 1: the contraction (taps x C1) is split four ways, one quarter per wavefront; every
//            wavefront accumulates a full R x 64 tile, then the four partial tiles are summed
//            through LDS.  Weights come straight from global memory in a pre-packed MFMA
//            fragment order (one coalesced 16-byte load per lane per fragment); the input
//            image is transposed into a zero-bordered, channels-last LDS tile per wavefront
//            so that a tap shift is a row offset.
//   stage 2: output channels are split across wavefronts; the intermediate is read from a
//            channels-last, zero-bordered LDS tile in bf16.
#pragma once

#include "pf_common.h"

namespace pf {

struct ChainArgs {
    const uint16_t *in;  // [N][C1][HW] bf16
    const uint4 *W1p;    // packed stage-1 weights, see make_pack_w1
    const uint4 *W2p;    // packed stage-2 weights, see make_pack_w2 (unused when W2nat is set)
    const uint16_t *W2nat; // 1x1 stage 2 only, nullable: weights in their natural [C2][R] layout (a lane per row:
                           // slow beyond a few output blocks; the fully connected mode at rank 64 uses it)
    uint16_t *out;       // [N][C2][HW] bf16
    uint16_t *mid_save;  // [N][R][HW] bf16, nullable
    int C1, C2, H, W;
    // fully connected ("channels last") mode only: in = X[rows][C1], out = Y[rows][C2], mid_save = T[rows][R]
    i64 rows;
    const void *bias; // bf16 [C2], nullable
    // Epilogue applied as the output is stored (image mode only; every member nullable / zero):
    //   out = mask > 0 ? act(scale[c] * out + shift[c] + add) : 0
    const float *ep_scale, *ep_shift; // float [C2], 16-byte aligned
    const uint16_t *ep_add;           // bf16 [N][C2][HW]: a residual input, or a gradient arriving over a skip connection
    const uint16_t *ep_mask;          // bf16 [N][C2][HW]: the output is zero where this is not positive
    int ep_relu;                      // act = max(0, .)
};

// Can the chain kernel take this problem?  (C1, C2: channels in / out of the chain.)
bool chain_supported(int C1, int C2, int R, int H, int W, int k, int stride, int pad);
size_t chain_w1_elems(int C1, int R, int k); // elements of the packed stage-1 weights
size_t chain_w2_elems(int C2, int R, int k); // elements of the packed stage-2 weights

// W1p[s][b][lane][e] = W1(rho = 32 b + lane % 32, c = 16 (s / T) + 8 (lane / 32) + e, tap = s % T)
// with W1(rho, c, tap) = src[rho * s_rho + c * s_c + tap * s_tap]; T = k * k.  src == NULL: nothing to pack.
struct PackW1 {
    const uint16_t *src;
    uint4 *dst;
    int n, RB, T; // n = number of 16-byte fragment slots
    i64 s_rho, s_c, s_tap;
    const float *cscale; // nullable: W1(rho, c, tap) is multiplied by cscale[c] (rounded to bf16 once more)
    // 0, or C1 / 4: the order the kernel wants for a 1x1 first stage of 7 x 7 images (chain_w1_interleaved): slot
    // s belongs to wavefront w = s / (C1 / 64), and k-step t of its round `sub` holds the channels
    // c = 256 sub + 4 (16 t + 8 (lane / 32) + e) + w instead of 16 s + 8 (lane / 32) + e.
    int il_cw;
};
bool chain_w1_interleaved(int k, int H, int W);
// W2p[ob][s2][lane][e] = W2(o = 32 ob + lane % 32, tap = s2 / (R / 16), rho = 16 (s2 % (R / 16)) + 8 (lane / 32) + e)
// with W2(o, tap, rho) = src[base + o * s_o + rho * s_rho + tap * s_tap].
struct PackW2 {
    const uint16_t *src;
    uint4 *dst;
    int n, S2, R16;
    i64 base, s_o, s_rho, s_tap;
};
// H, W: image size of the chain kernel that will read the weights (0, 0 for the fully connected mode)
PackW1 make_pack_w1(const uint16_t *src, uint4 *dst, int C1, int R, int k, i64 s_rho, i64 s_c, i64 s_tap, int H = 0, int W = 0);
PackW2 make_pack_w2(const uint16_t *src, uint4 *dst, int C2, int R, int k, i64 base, i64 s_o, i64 s_rho, i64 s_tap);
int launch_pack_chain(hipStream_t s, const PackW1 &p1, const PackW2 &p2, const PackW1 &p3 = PackW1{},
                      const PackW2 &p4 = PackW2{});
// The fully connected layer on the same kernel: Y[rows][C2] = (X[rows][C1] W1^T) W2^T + bias, W2 = a.W2nat.
bool linear_chain_supported(i64 n_in, i64 n_out, i64 r);
int launch_linear_chain(hipStream_t s, const char *name, const ChainArgs &a, int R);
// k1 / k2: kernel sizes of the two stages (1 or 3); R: 64 or 128.
int launch_conv_chain(hipStream_t s, const char *name, const ChainArgs &a, int N, int k1, int k2, int R);

} // namespace pf
