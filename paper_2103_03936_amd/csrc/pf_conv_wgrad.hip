// Filter-gradient kernel for small images (bf16 in, fp32 accumulate), stride 1, "same" geometry:
//     Out[m][n][tap] = sum_{img, y, x}  A[img][m][y][x] * Bpad[img][n][y + ty - 1][x + tx - 1]
// with tap = 3 ty + tx for a 3x3 stage, or a single tap (no shift) for a 1x1 stage.
//     dUk (Section 2.2 backward, thin k x k stage):  A = dT  (m = rank index), B = X  (n = input channel)
//     dVp (1x1 stage), computed transposed:          A = T   (m = rank index), B = dY (n = output channel)
//
// The contraction runs over pixels.  An image row of up to 8 pixels is one 8-element MFMA
// k-fragment (x >= W reads as zero), two rows make one 32x32x16 k-step.  Each workgroup owns a
// slab of B channels (all taps) and a group of images; it writes one partial sum per group,
// laid out [tap][m][n] so that stores are coalesced; pf_wgrad_reduce sums the groups and puts
// the result where the caller's layout wants it.
//
// For a 3x3 stage the B rows are staged in LDS three times, shifted by tx - 1 with the zero
// border baked in, so every fragment read is an aligned 16-byte LDS load; A fragments and 1x1
// B fragments come straight from global memory.
#include "pf_conv_wgrad.h"

namespace pf {

constexpr int WG_ROWS = 11; // LDS rows per channel: 1 zero row above, up to 8 rows, zero rows below (pitch 176 B)

typedef uint4 __attribute__((may_alias)) uint4_alias;

__device__ __forceinline__ bf16x8_t wg_as_bf16x8(uint4 v)
{
    union {
        uint4 u;
        bf16x8_t b;
    } c;
    c.u = v;
    return c.b;
}

// Row y of one channel plane (W <= 8 pixels) as 8 bf16, zero beyond W and for y >= H; branch-free so that
// many row loads can be in flight at once.  `plane` points at the channel's first pixel.  Rows of 8-pixel
// images are 16-byte aligned; other widths are read element by element (indices clamped into the row).
struct __attribute__((packed, aligned(2))) U16x8 {
    uint16_t v[8];
};

template <int WC>
__device__ __forceinline__ uint4 load_row(const uint16_t *plane, int y, int H, int W)
{
    const int yy = y < H ? y : H - 1;
    uint4 v;
    if (WC == 8) {
        v = *(const uint4 *)(plane + 8 * yy);
    } else if (WC == 7) {
        // A row is 14 bytes at a 2-byte aligned address: one unaligned 16-byte load.  It reaches one element
        // past the row, so the last row (H >= 2) is read one element early and shifted down, which keeps the
        // load inside the plane.
        const bool last = yy == H - 1;
        const U16x8 t = *(const U16x8 *)(plane + 7 * yy - (last ? 1 : 0));
        const uint32_t w0 = t.v[0] | ((uint32_t)t.v[1] << 16), w1 = t.v[2] | ((uint32_t)t.v[3] << 16),
                       w2 = t.v[4] | ((uint32_t)t.v[5] << 16), w3 = t.v[6] | ((uint32_t)t.v[7] << 16);
        v = last ? make_uint4((w0 >> 16) | (w1 << 16), (w1 >> 16) | (w2 << 16), (w2 >> 16) | (w3 << 16), w3 >> 16)
                 : make_uint4(w0, w1, w2, w3 & 0xffffu);
    } else {
        const uint16_t *p = plane + W * yy;
        uint32_t e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t x = p[i < W ? i : W - 1];
            e[i] = i < W ? x : 0u;
        }
        v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
    const bool ok = y < H;
    return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
}

// TAPS: 9 (3x3, pad 1) or 1.  MB: 32-row blocks of m (M = 32 MB).  NBLK: 32-channel blocks of n per workgroup.
// Pairs (n-block, tap) are dealt to the four wavefronts round-robin; PW = pairs per wavefront (max).
// HC, WC: image height / width known at compile time (0 = read them from the arguments).
template <int TAPS, int MB, int NBLK, int HC, int WC>
__device__ __forceinline__ void conv_wgrad_body(const WgradArgs &a, const int bx, const int g)
{
    constexpr int NPAIR = NBLK * TAPS;
    constexpr int PW = (NPAIR + 3) / 4;
    constexpr int NCH = 32 * NBLK;
    constexpr int LDS_ELEMS = TAPS == 9 ? 2 * 3 * NCH * WG_ROWS * 8 : 8;
    __shared__ __attribute__((aligned(16))) uint16_t Xsh[LDS_ELEMS]; // [buf][tx][channel][row][8]
    // The A fragments of an image are the same for all four wavefronts.  Each fetches a quarter (k-step j = its
    // own index, all m blocks) and they trade through LDS: a lane-per-row fragment load costs the L1 one cache
    // line per lane, an LDS read of the finished fragment 16 bytes.
    constexpr bool SHARE_A = true;
    __shared__ __attribute__((aligned(16))) uint4 Ash[SHARE_A ? 2 * MB * 4 * 64 : 1]; // [buf][m block][k-step][lane]

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int H = HC ? HC : a.H, W = WC ? WC : a.W, HW = H * W, M = 32 * MB;
    const int n0 = bx * NCH; // first B channel of this workgroup
    const int img0 = g * a.imgs_per_group;
    const int img1 = min(a.N_img, img0 + a.imgs_per_group);
    const int ksteps = (H + 1) / 2;

    if (TAPS == 9) { // zero both buffers once: border rows and unused rows stay zero
        uint4_alias *z = (uint4_alias *)Xsh;
        for (int i = tid; i < LDS_ELEMS / 8; i += 256) z[i] = make_uint4(0, 0, 0, 0);
    }

    f32x16_t acc[MB][PW];
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int p = 0; p < PW; ++p)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][p][v] = 0.f;

    // Everything one image needs from global memory, fetched two images ahead of its staging:
    // the rows of B this thread stages (3x3) or this lane's B fragments (1x1), and this wavefront's share of
    // the A fragments (k-step w of every m block).
    constexpr int ROWS_PT = TAPS == 9 ? (NCH * 8 + 255) / 256 : 1;
    constexpr int NBF = TAPS == 9 ? 1 : PW;
    struct Stage {
        uint4 brow[ROWS_PT];
        uint4 bfr[NBF][4];
        uint4 afr[MB];
    };
    auto load_image = [&](Stage &st, int img) __attribute__((always_inline)) {
        if (img >= img1) return;
        if (TAPS == 9) {
#pragma unroll
            for (int i = 0; i < ROWS_PT; ++i) {
                const int item = tid + 256 * i, c = item >> 3, y = item & 7;
                st.brow[i] = load_row<WC>(a.B + ((i64)img * a.Nc + n0 + c) * HW, y, H, W);
            }
        } else {
#pragma unroll
            for (int p = 0; p < PW; ++p)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int y = 2 * j + half, pair = w + 4 * p;
                    const int ch = n0 + 32 * (pair < NPAIR ? pair : 0) + col;
                    st.bfr[p][j] = load_row<WC>(a.B + ((i64)img * a.Nc + ch) * HW, y, H, W);
                }
        }
#pragma unroll
        for (int b = 0; b < MB; ++b)
            st.afr[b] = load_row<WC>(a.A + ((i64)img * M + 32 * b + col) * HW, 2 * w + half, H, W);
    };
    // The image held in st goes to LDS buffer `buf` (A fragments; for 3x3 the three shifted copies of this
    // thread's B rows); 1x1 B fragments stay in registers (bnext) until their image is multiplied.
    uint4 bnext[NBF][4];
    auto stage_to_lds = [&](const Stage &st, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < MB; ++b) *(uint4_alias *)&Ash[((buf * MB + b) * 4 + w) * 64 + lane] = st.afr[b];
#pragma unroll
        for (int p = 0; p < NBF; ++p)
#pragma unroll
            for (int j = 0; j < 4; ++j) bnext[p][j] = st.bfr[p][j];
        if (TAPS == 9) {
#pragma unroll
            for (int i = 0; i < ROWS_PT; ++i) {
                const int item = tid + 256 * i, c = item >> 3, y = item & 7;
                if (y < H) {
                    const uint4 r = st.brow[i];
                    // tx = 0 reads x - 1: shift towards higher x, zero enters at x = 0
                    const uint4 s0 = make_uint4(r.x << 16, (r.y << 16) | (r.x >> 16), (r.z << 16) | (r.y >> 16),
                                                (r.w << 16) | (r.z >> 16));
                    // tx = 2 reads x + 1: shift towards lower x, zero enters at x = 7
                    const uint4 s2 = make_uint4((r.x >> 16) | (r.y << 16), (r.y >> 16) | (r.z << 16),
                                                (r.z >> 16) | (r.w << 16), r.w >> 16);
                    uint16_t *base = &Xsh[((buf * 3) * NCH + c) * WG_ROWS * 8 + (y + 1) * 8];
                    *(uint4_alias *)(base) = s0;
                    *(uint4_alias *)(base + NCH * WG_ROWS * 8) = r;
                    *(uint4_alias *)(base + 2 * NCH * WG_ROWS * 8) = s2;
                }
            }
        }
    };
    // One image: its fragments come out of LDS buffer `buf` into registers; then the next image (in st) is
    // staged into the other buffer and st refilled two images further on, so that those LDS writes, the global
    // requests and the barrier's wait overlap this image's MFMAs, which only need registers.
    auto step = [&](Stage &st, int img, int buf) __attribute__((always_inline)) {
        uint4 acur[MB][4], bcur[PW][4];
#pragma unroll
        for (int b = 0; b < MB; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j) acur[b][j] = *(const uint4_alias *)&Ash[((buf * MB + b) * 4 + j) * 64 + lane];
#pragma unroll
        for (int p = 0; p < PW; ++p) {
            const int pair = w + 4 * p;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (TAPS == 9) {
                    const int pr = pair < NPAIR ? pair : 0, nb = pr / TAPS, tap = pr % TAPS;
                    const int ty = tap / 3, tx = tap % 3;
                    bcur[p][j] = *(const uint4_alias *)&Xsh[((buf * 3 + tx) * NCH + 32 * nb + col) * WG_ROWS * 8 +
                                                            (2 * j + half + ty) * 8];
                } else {
                    bcur[p][j] = bnext[p < NBF ? p : 0][j];
                }
            }
        }
        if (img + 1 < img1) stage_to_lds(st, buf ^ 1); // (uniform)
        load_image(st, img + 3);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j >= ksteps) break;
#pragma unroll
            for (int p = 0; p < PW; ++p) {
                if (w + 4 * p < NPAIR) {
#pragma unroll
                    for (int b = 0; b < MB; ++b)
                        acc[b][p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg_as_bf16x8(acur[b][j]),
                                                                            wg_as_bf16x8(bcur[p][j]), acc[b][p], 0, 0, 0);
                }
            }
        }
        __syncthreads(); // the staged image is complete; the buffer just read may be rewritten
    };

    if (img0 < img1) { // (uniform; an empty group writes zeros below)
        Stage sA, sB;
        load_image(sA, img0);
        load_image(sB, img0 + 1);
        __syncthreads(); // the zero fill above
        stage_to_lds(sA, 0);
        load_image(sA, img0 + 2);
        __syncthreads();
        for (int img = img0; img < img1; img += 2) {
            step(sB, img, 0);
            if (img + 1 < img1) step(sA, img + 1, 1);
        }
    }

    // partial[g][tap][m][n]
    float *part = a.partial + (i64)g * TAPS * M * a.Nc;
#pragma unroll
    for (int p = 0; p < PW; ++p) {
        const int pair = w + 4 * p;
        if (pair < NPAIR) {
            const int nb = pair / TAPS, tap = pair % TAPS;
#pragma unroll
            for (int b = 0; b < MB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = 32 * b + 8 * (v >> 2) + 4 * half + (v & 3);
                    part[((i64)tap * M + m) * a.Nc + n0 + 32 * nb + col] = acc[b][p][v];
                }
        }
    }
}

// One launch computes both filter gradients: the first nwg1 workgroups work on problem 1 (taps T1: the
// k x k stage), the others on problem 2 (always a 1x1 stage).  Each problem has its own image grouping.
template <int T1, int MB, int HC, int WC>
__global__ __launch_bounds__(256, 1) void conv_wgrad_pair_kernel(WgradArgs a1, WgradArgs a2, int nx1, int nx2, int nwg1)
{
    const int b = blockIdx.x;
    if (b < nwg1)
        conv_wgrad_body<T1, MB, (T1 == 9 ? 1 : 8), HC, WC>(a1, b % nx1, b / nx1);
    else
        conv_wgrad_body<1, MB, 4, HC, WC>(a2, (b - nwg1) % nx2, (b - nwg1) / nx2);
}

// out[m * s_m + n * s_n + tap * s_tap] (+)= sum_g partial[g][tap][m][n]; four consecutive n per thread
// The blocks past blocks01 add up per-tile column sums instead (a bias gradient): 32 columns per block,
// eight threads per column take every eighth tile, and their sums are added in a fixed order.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(WgradReduceArgs r0, WgradReduceArgs r1, int blocks0,
                                                            ColsumTilesArgs cs, int blocks01)
{
    if ((int)blockIdx.x >= blocks01) {
        __shared__ float part[8][32];
        const int tc = threadIdx.x & 31, tg = threadIdx.x >> 5;
        const int colm = (blockIdx.x - blocks01) * 32 + tc;
        const float *p = cs.partial + colm;
        float acc = 0.f;
        int t = tg;
        for (; t + 56 < cs.tiles; t += 64) { // eight loads in flight
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = p[(i64)(t + 8 * u) * cs.cols];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; t < cs.tiles; t += 8) acc += p[(i64)t * cs.cols];
        part[tg][tc] = acc;
        __syncthreads();
        if (tg == 0) {
            float sum = 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) sum += part[u][tc];
            cs.out[colm] = cs.accumulate ? cs.out[colm] + sum : sum;
        }
        return;
    }
    const bool second = (int)blockIdx.x >= blocks0;
    const WgradReduceArgs r = second ? r1 : r0;
    const i64 i4 = (i64)(blockIdx.x - (second ? blocks0 : 0)) * 256 + threadIdx.x;
    const i64 count = (i64)r.taps * r.M * r.Nc; // multiple of 4: Nc is a multiple of 32
    if (4 * i4 >= count) return;
    const float4 *p = (const float4 *)r.partial + i4;
    const i64 stride4 = count / 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    int g = 0;
    for (; g + 8 <= r.groups; g += 8) { // eight independent loads in flight, summed in group order
        float4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = p[(i64)(g + k) * stride4];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            s.x += v[k].x;
            s.y += v[k].y;
            s.z += v[k].z;
            s.w += v[k].w;
        }
    }
    for (; g < r.groups; ++g) {
        const float4 v = p[(i64)g * stride4];
        s.x += v.x;
        s.y += v.y;
        s.z += v.z;
        s.w += v.w;
    }
    const i64 i = 4 * i4;
    const int n = (int)(i % r.Nc);
    const i64 t = i / r.Nc;
    const int m = (int)(t % r.M), tap = (int)(t / r.M);
    float *dst = r.out + m * r.s_m + n * r.s_n + tap * r.s_tap;
    const float v[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) dst[e * r.s_n] = r.accumulate ? (dst[e * r.s_n] + v[e]) : v[e];
}

bool wgrad_supported(int M, int Nc, int H, int W, int k, int stride, int pad)
{
    if (stride != 1) return false;
    if (!((k == 3 && pad == 1) || (k == 1 && pad == 0))) return false;
    if (H > 8 || W > 8) return false;
    if (M != 64 && M != 128) return false;
    return Nc % 256 == 0;
}

int wgrad_nchunk(int M, int k, int which)
{
    (void)M;
    if (which == 2) return 128; // the 1x1 stage as second problem of a pair
    return k == 3 ? 32 : 256;
}

// a1: the k x k stage (k = 3 or 1); a2: the 1x1 stage; either may be skipped by passing partial == NULL.
int launch_conv_wgrad_pair(hipStream_t s, const WgradArgs &a1, int k1, const WgradArgs &a2)
{
    int st = PF_OK;
    if (a1.N_img <= 0) return st;
    const int nx1 = a1.partial ? a1.Nc / wgrad_nchunk(a1.M, k1, 1) : 0;
    const int nx2 = a2.partial ? a2.Nc / wgrad_nchunk(a2.M, 1, 2) : 0;
    const int nwg1 = nx1 * a1.groups, nwg2 = nx2 * a2.groups;
    if (nwg1 + nwg2 == 0) return st;
    const dim3 grid(nwg1 + nwg2), block(256);
    const int M = a1.M, x1 = nx1 > 0 ? nx1 : 1, x2 = nx2 > 0 ? nx2 : 1;
    const bool sq8 = a1.H == 8 && a1.W == 8, sq7 = a1.H == 7 && a1.W == 7;
#define PF_WGRAD_CASE(T1, MBV)                                                                                     \
    if (k1 * k1 == T1 && M == 32 * MBV) {                                                                          \
        if (sq8) {                                                                                                 \
            PF_LAUNCH(st, "conv_wgrad_pair", (conv_wgrad_pair_kernel<T1, MBV, 8, 8>), grid, block, s, a1, a2, x1,  \
                      x2, nwg1);                                                                                   \
        } else if (sq7) {                                                                                          \
            PF_LAUNCH(st, "conv_wgrad_pair", (conv_wgrad_pair_kernel<T1, MBV, 7, 7>), grid, block, s, a1, a2, x1,  \
                      x2, nwg1);                                                                                   \
        } else {                                                                                                   \
            PF_LAUNCH(st, "conv_wgrad_pair", (conv_wgrad_pair_kernel<T1, MBV, 0, 0>), grid, block, s, a1, a2, x1,  \
                      x2, nwg1);                                                                                   \
        }                                                                                                          \
        return st;                                                                                                 \
    }
    PF_WGRAD_CASE(9, 2)
    PF_WGRAD_CASE(9, 4)
    PF_WGRAD_CASE(1, 2)
    PF_WGRAD_CASE(1, 4)
#undef PF_WGRAD_CASE
    return PF_ERR_UNSUPPORTED;
}

int launch_wgrad_reduce(hipStream_t s, const WgradReduceArgs &r0, const WgradReduceArgs &r1, const ColsumTilesArgs *cs)
{
    int st = PF_OK;
    const i64 c0 = r0.out ? (i64)r0.taps * r0.M * r0.Nc : 0, c1 = r1.out ? (i64)r1.taps * r1.M * r1.Nc : 0;
    const int b0 = (int)((c0 / 4 + 255) / 256), b1 = (int)((c1 / 4 + 255) / 256);
    ColsumTilesArgs c = {};
    if (cs && cs->out && cs->tiles > 0) c = *cs;
    if (c.cols % 32 != 0) return PF_ERR_UNSUPPORTED;
    const int b2 = c.cols / 32;
    if (b0 + b1 + b2 == 0) return st;
    PF_LAUNCH(st, "wgrad_reduce", wgrad_reduce_kernel, dim3(b0 + b1 + b2), dim3(256), s, r0, r1, b0, c, b0 + b1);
    return st;
}

} // namespace pf
