// Factor gradients of the fully connected layer (bf16 in, fp32 accumulate):
//     dU^T[rho][o] = sum_rows T[row][rho]  * dY[row][o]        (Section 2.1 backward)
//     dV^T[rho][i] = sum_rows dT[row][rho] * X[row][i]
// Both are "TN" products: the contraction runs over rows, which is the slow index of both row-major
// operands, while a bf16 MFMA wants 8 consecutive k per lane.  Tiles of 64 rows are copied to LDS as they
// are (coalesced 16-byte loads, 16-byte LDS writes) and the fragments are fetched with the transposing LDS
// read ds_read_b64_tr_b16: within each group of 16 lanes, lane 4 q + c receives element c of the 8-byte
// chunks addressed by lanes q, q + 4, q + 8, q + 12.  Pointing lane q + 4 e at &tile[m0 + e][c0 + 4 q]
// therefore hands lane i the four rows m0 .. m0 + 3 of column c0 + i; two such reads make one fragment.
//
// A workgroup owns 256 columns of B (all of rho) and a group of row tiles; it writes one fp32 partial sum
// [group][rho][column]; wgrad_reduce_kernel adds the groups in a fixed order.
#include "pf_conv_wgrad.h"

namespace pf {

typedef uint4 __attribute__((may_alias)) uint4_alias;
constexpr int LW_ROWS = 64;  // rows per tile

// MB: 32-row blocks of rho (M = 32 MB = the rank, 64 or 128).  LW_COLS: B columns per workgroup, 256 or 128
// (the narrower tile doubles the number of workgroups when the layer is small).
template <int MB, int LW_COLS>
__global__ __launch_bounds__(256, 1) void linear_wgrad_pair_kernel(WgradArgs a1, WgradArgs a2, int nx1, int nx2, int nwg1)
{
    // Both factor gradients in one launch: problem 1 in the first nwg1 workgroups, problem 2 in the rest.
    const bool first = (int)blockIdx.x < nwg1;
    const WgradArgs &a = first ? a1 : a2;
    const int bidx = first ? blockIdx.x : blockIdx.x - nwg1, nx = first ? nx1 : nx2;
    const int bx = bidx % nx, g = bidx / nx;
    constexpr int M = 32 * MB;
    constexpr int AP = M + 16;          // LDS row pitch of the A tile (288 or 160 bytes: 32 mod 128)
    constexpr int LW_BP = LW_COLS + 16; // LDS row pitch (elements) of the B tile: 32 bytes mod 128
    constexpr int RW = 2;               // rho blocks per wavefront
    constexpr int CW = (LW_COLS / 32) * MB / 8; // column blocks per wavefront (MB x LW_COLS / 32 blocks over 4 wavefronts)
    constexpr int AV = LW_ROWS * M / 8 / 256;       // 16-byte vectors of the A tile per thread (4 or 2)
    constexpr int BV = LW_ROWS * LW_COLS / 8 / 256; // of the B tile (8)
    __shared__ __attribute__((aligned(16))) uint16_t As[2][LW_ROWS * AP];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][LW_ROWS * LW_BP];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int n0 = bx * LW_COLS;
    const int rb0 = RW * (w % (MB / RW)), cb0 = CW * (w / (MB / RW)); // this wavefront's first rho / column block
    const int t0 = g * a.imgs_per_group, t1 = min(a.N_img, t0 + a.imgs_per_group);

    f32x16_t acc[RW][CW];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int c = 0; c < CW; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

    // Two register sets hold the tiles that are in flight from global memory (two tiles ahead of the MFMAs),
    // two LDS buffers hold the tile being multiplied and the one being written.
    struct Regs {
        uint4 av[AV], bv[BV];
    };
    // tile t: rows 64 t ..; rows past the end re-read the last row, and read as zero on the A side
    auto load_tile = [&](Regs &rg, int t) __attribute__((always_inline)) {
        if (t >= t1) return;
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int it = tid + 256 * i, m = it / (M / 8), o = it % (M / 8);
            const i64 row = (i64)t * LW_ROWS + m;
            const uint4 v = *(const uint4 *)(a.A + (row < a.rows ? row : a.rows - 1) * M + 8 * o);
            const bool ok = row < a.rows;
            rg.av[i] = make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            const int it = tid + 256 * i, m = it / (LW_COLS / 8), o = it % (LW_COLS / 8);
            const i64 row = (i64)t * LW_ROWS + m;
            rg.bv[i] = *(const uint4 *)(a.B + (row < a.rows ? row : a.rows - 1) * a.Nc + n0 + 8 * o);
        }
    };
    // write the tile held in rg to LDS buffer `buf`, refill rg with tile t + 2, then multiply out of `buf`
    auto step = [&](Regs &rg, int t, int buf) __attribute__((always_inline)) {
        if (t >= t1) return;
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int it = tid + 256 * i, m = it / (M / 8), o = it % (M / 8);
            *(uint4_alias *)&As[buf][m * AP + 8 * o] = rg.av[i];
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            const int it = tid + 256 * i, m = it / (LW_COLS / 8), o = it % (LW_COLS / 8);
            *(uint4_alias *)&Bs[buf][m * LW_BP + 8 * o] = rg.bv[i];
        }
        load_tile(rg, t + 2);
        __syncthreads(); // one barrier per tile: the buffer rewritten next time was last read two tiles ago
#pragma unroll
        for (int j = 0; j < LW_ROWS / 16; ++j) {
            bf16x8_t af[RW], bf[CW];
#pragma unroll
            for (int r = 0; r < RW; ++r) af[r] = lds_frag_tr(&As[buf][0], AP, 16 * j, 32 * (rb0 + r), lane);
#pragma unroll
            for (int c = 0; c < CW; ++c) bf[c] = lds_frag_tr(&Bs[buf][0], LW_BP, 16 * j, 32 * (cb0 + c), lane);
#pragma unroll
            for (int r = 0; r < RW; ++r)
#pragma unroll
                for (int c = 0; c < CW; ++c) acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[r], bf[c], acc[r][c], 0, 0, 0);
        }
    };

    Regs r0, r1;
    load_tile(r0, t0);
    load_tile(r1, t0 + 1);
    for (int t = t0; t < t1; t += 2) {
        step(r0, t, 0);
        step(r1, t + 1, 1);
    }

    // partial[g][rho][column]
    float *part = a.partial + (i64)g * M * a.Nc;
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int c = 0; c < CW; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rho = 32 * (rb0 + r) + 8 * (v >> 2) + 4 * half + (v & 3);
                part[(i64)rho * a.Nc + n0 + 32 * (cb0 + c) + col] = acc[r][c][v];
            }
}

// a1, a2: A[rows][M], B[rows][Nc] row-major bf16, N_img = number of 64-row tiles, Nc a multiple of 256,
// M = 64 or 128; partial == NULL skips a problem.  cols: B columns per workgroup, 256 or 128.
int launch_linear_wgrad_pair(hipStream_t s, const WgradArgs &a1, const WgradArgs &a2, int cols)
{
    int st = PF_OK;
    if (a1.N_img <= 0) return st;
    if (cols != 256 && cols != 128) return PF_ERR_UNSUPPORTED;
    const int nx1 = a1.partial ? a1.Nc / cols : 0, nx2 = a2.partial ? a2.Nc / cols : 0;
    const int nwg1 = nx1 * a1.groups, nwg2 = nx2 * a2.groups;
    if (nwg1 + nwg2 == 0) return st;
    const dim3 grid(nwg1 + nwg2), block(256);
    const int x1 = nx1 > 0 ? nx1 : 1, x2 = nx2 > 0 ? nx2 : 1;
    if (a1.M == 64 && cols == 256) {
        PF_LAUNCH(st, "linear_wgrad_pair", (linear_wgrad_pair_kernel<2, 256>), grid, block, s, a1, a2, x1, x2, nwg1);
    } else if (a1.M == 64) {
        PF_LAUNCH(st, "linear_wgrad_pair", (linear_wgrad_pair_kernel<2, 128>), grid, block, s, a1, a2, x1, x2, nwg1);
    } else if (a1.M == 128 && cols == 256) {
        PF_LAUNCH(st, "linear_wgrad_pair", (linear_wgrad_pair_kernel<4, 256>), grid, block, s, a1, a2, x1, x2, nwg1);
    } else if (a1.M == 128) {
        PF_LAUNCH(st, "linear_wgrad_pair", (linear_wgrad_pair_kernel<4, 128>), grid, block, s, a1, a2, x1, x2, nwg1);
    } else {
        st = PF_ERR_UNSUPPORTED;
    }
    return st;
}

} // namespace pf
