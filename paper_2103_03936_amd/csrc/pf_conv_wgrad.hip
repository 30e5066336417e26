// Filter-gradient kernel for small images (bf16 in, fp32 accumulate), stride 1, "same" geometry:
//     Out[m][n][tap] = sum_{img, y, x}  A[img][m][y][x] * Bpad[img][n][y + ty - 1][x + tx - 1]
// with tap = 3 ty + tx for a 3x3 stage, or a single tap (no shift) for a 1x1 stage.
//     dUk (Section 2.2 backward, thin k x k stage):  A = dT  (m = rank index), B = X  (n = input channel)
//     dVp (1x1 stage), computed transposed:          A = T   (m = rank index), B = dY (n = output channel)
//
// The contraction runs over pixels, 16 per MFMA k-step: two image rows of 8 pixel slots (x >= W reads as
// zero) for a 3x3 stage, 16 consecutive pixels for a 1x1 stage.  Each workgroup owns a slab of B channels (all
// taps), 64 or 128 rows of A, and a group of images; it writes one partial sum per group, laid out [tap][m][n]
// so that stores are coalesced; wgrad_reduce_kernel sums the groups and puts the result where the caller's
// layout wants it.
//
// Everything is fetched from global memory in memory order (a lane-per-row fragment load costs the L1 one
// cache line per lane), several images ahead, and laid out in LDS with 64 pixel slots per plane so that every
// MFMA fragment is one aligned 16-byte LDS read.  For a 3x3 stage the B rows are staged three times, shifted
// by tx - 1 with the zero border baked in.
#include "pf_conv_wgrad.h"

namespace pf {

constexpr int WG_THREADS = 512; // of the filter-gradient kernel
constexpr int WG_ND = 4;        // images it keeps in flight from global memory (even)
constexpr int WG_ROWS = 11; // LDS rows per channel: 1 zero row above, up to 8 rows, zero rows below (pitch 176 B)

typedef uint4 __attribute__((may_alias)) uint4_alias;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4))); // plain vector: stays in registers inside arrays
typedef u32x4 __attribute__((may_alias)) u32x4_alias;
__device__ __forceinline__ bf16x8_t wg_bf(u32x4 v) { return __builtin_bit_cast(bf16x8_t, v); }

// Row y of one channel plane (W <= 8 pixels) as 8 bf16, zero beyond W and for y >= H, in two parts: row_fetch
// issues the load (branch-free, indices clamped, so that many stay in flight) and row_fix, called when the data
// is needed, puts the pixels in place.  `plane` points at the channel's first pixel.  Rows of 8-pixel images
// are 16-byte aligned.  A row of a 7-pixel image is 14 bytes at a 2-byte aligned address and is fetched with
// one unaligned 16-byte load; that reaches one element past the row, so the last row (H >= 2) is read one
// element early and shifted down afterwards, which keeps the load inside the plane.  Other widths are read
// element by element.
typedef u32x4 __attribute__((aligned(2))) u32x4_a2;

template <int WC>
__device__ __forceinline__ u32x4 row_fetch(const uint16_t *plane, int y, int H, int W)
{
    const int yy = y < H ? y : H - 1;
    if (WC == 8) return *(const u32x4 *)(plane + 8 * yy);
    if (WC == 7) return *(const u32x4_a2 *)(plane + 7 * yy - (yy == H - 1 ? 1 : 0));
    const uint16_t *p = plane + W * yy;
    uint32_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t x = p[i < W ? i : W - 1];
        e[i] = i < W ? x : 0u;
    }
    return u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
}

template <int WC>
__device__ __forceinline__ u32x4 row_fix(u32x4 v, int y, int H)
{
    if (WC == 7) {
        const bool last = y >= H - 1;
        v = last ? u32x4{(v.x >> 16) | (v.y << 16), (v.y >> 16) | (v.z << 16), (v.z >> 16) | (v.w << 16), v.w >> 16}
                 : u32x4{v.x, v.y, v.z, v.w & 0xffffu};
    }
    return y < H ? v : u32x4{0u, 0u, 0u, 0u};
}

// Compile-time shape of one problem.  TAPS: 9 (3x3, pad 1) or 1.  MB: 32-row blocks of m (M = 32 MB).  NBLK:
// 32-channel blocks of n per workgroup.  HC, WC: image height / width (0 = read them from the arguments).
//
// Eight wavefronts (two per SIMD, so that one multiplies while the other waits for LDS or the barrier) split
// an image three ways.  kh = w & 1 takes k-steps 2 kh, 2 kh + 1 (image rows 4 kh .. 4 kh + 3, or pixels
// 32 kh .. 32 kh + 31 of a 1x1 stage); the other four pairs of wavefronts split the m blocks in two (when there
// are at least two) and the (n block, tap) pairs in two or four.  At the end the two k halves trade half of their tiles through LDS, add, and each
// stores the half it kept.
template <int TAPS, int MB, int NBLK, int HC, int WC>
struct WgCfg {
    static constexpr int M = 32 * MB, NCH = 32 * NBLK, NPAIR = NBLK * TAPS;
    static constexpr int MQ = MB >= 2 ? 2 : 1, PQ = 4 / MQ; // ways the m blocks / the pairs are split
    static constexpr int MBW = MB / MQ;                     // m blocks per wavefront
    static constexpr int PWN = (NPAIR + PQ - 1) / PQ;       // pairs per wavefront
    static constexpr int TILES = MBW * PWN, KEEP = (TILES + 1) / 2;
    static constexpr bool AL8 = HC == 8 && WC == 8; // planes of 64 pixels: rows are aligned 16-byte pieces
    // LDS copies of the A block / B slab of one image: 64 pixel slots per plane, plane pitch 144 bytes (against
    // bank conflicts); a 3x3 stage keeps its B slab as three shifted copies with zero borders instead
    static constexpr int A_BYTES = M * 144;
    static constexpr int B_BYTES = TAPS == 9 ? 3 * NCH * WG_ROWS * 16 : NCH * 144;
    static constexpr int STAGE_BYTES = 2 * (A_BYTES + B_BYTES);
    static constexpr int RED_BYTES = (WG_THREADS / 64) * KEEP * 4096;
    static constexpr int LDS_BYTES = STAGE_BYTES > RED_BYTES ? STAGE_BYTES : RED_BYTES;
    // images in flight from global memory (even): enough to cover the memory latency at about a thousand
    // cycles per image, within the registers left beside the accumulators
    static constexpr int ND = WG_ND;
};

template <int TAPS, int MB, int NBLK, int HC, int WC>
__device__ __forceinline__ void conv_wgrad_body(const WgradArgs &a, const int bx, const int g, const int m_off,
                                                unsigned char *lds)
{
    typedef WgCfg<TAPS, MB, NBLK, HC, WC> C;
    constexpr int M = C::M, NCH = C::NCH, NPAIR = C::NPAIR, MBW = C::MBW, PWN = C::PWN, ND = C::ND;
    constexpr bool AL8 = C::AL8;
    static_assert(TAPS == 1 || NBLK == 1, "a 3x3 workgroup stages one 32-channel block");

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int kh = w & 1, mb0 = MBW * ((w >> 1) % C::MQ), p0 = PWN * ((w >> 1) / C::MQ);
    const int H = HC ? HC : a.H, W = WC ? WC : a.W, HW = H * W;
    const int n0 = bx * NCH; // first B channel of this workgroup
    const int img0 = g * a.imgs_per_group;
    const int img1 = min(a.N_img, img0 + a.imgs_per_group);
    constexpr bool SQ7 = HC == 7 && WC == 7 && TAPS == 9;
    // 16-byte items of the A block / the B slab of one image (7x7: one per 8-pixel slot group of a plane)
    const int apieces = SQ7 ? M * 7 : M * HW / 8, bpieces = SQ7 ? NCH * 7 : NCH * HW / 8;
    constexpr int NT = WG_THREADS;
    constexpr int APT = (MB * 256 + NT - 1) / NT, BPT = TAPS == 9 ? 1 : NBLK * 256 / NT; // items per thread (at most)

    auto a_buf = [&](int buf) __attribute__((always_inline)) { return lds + buf * (C::A_BYTES + C::B_BYTES); };
    auto b_buf = [&](int buf) __attribute__((always_inline)) { return a_buf(buf) + C::A_BYTES; };

    if (TAPS == 9 || !AL8) { // zero the staging buffers once: borders, unused rows and pixel slots stay zero
        uint4_alias *z = (uint4_alias *)lds;
        for (int i = tid; i < C::STAGE_BYTES / 16; i += NT) z[i] = make_uint4(0, 0, 0, 0);
    }

    f32x16_t acc[MBW][PWN];
#pragma unroll
    for (int b = 0; b < MBW; ++b)
#pragma unroll
        for (int p = 0; p < PWN; ++p)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][p][v] = 0.f;

    // What one image needs from global memory: the A block and (1x1) the B slab as 16-byte items in memory
    // order, (3x3) one row of the B slab per thread.  Loads are unconditional (indices clamped) so that several
    // images stay in flight.  8x8 and other shapes: item = aligned piece of the planes laid end to end.  7x7:
    // item (plane, c) = the 8 elements that fill slots 8 c .. 8 c + 7 of the plane's LDS copy, one unaligned
    // load: row c of the image (3x3) or pixels 8 c .. 8 c + 7 (1x1); the last item of a plane is read from
    // further back so that it stays inside the plane, and shifted when it is stored.
    struct Stage {
        u32x4 av[APT], bv[BPT];
    };
    auto fetch_item = [&](const uint16_t *base, int it) __attribute__((always_inline)) {
        if (SQ7) {
            const int plane = it / 7, c = it - 7 * plane;
            const int off = TAPS == 9 ? 7 * c - (c == 6 ? 1 : 0) : 8 * c - (c == 6 ? 7 : 0);
            return (u32x4) * (const u32x4_a2 *)(base + 49 * plane + off);
        }
        return *(const u32x4 *)(base + 8 * it);
    };
    auto load_image = [&](Stage &st, int img) __attribute__((always_inline)) {
        const int im = img < img1 ? img : img1 - 1;
        const uint16_t *Ab = a.A + ((i64)im * a.M + m_off) * HW; // M planes of the a.M, from m_off on
#pragma unroll
        for (int i = 0; i < APT; ++i) {
            const int pc = tid + NT * i;
            st.av[i] = fetch_item(Ab, pc < apieces ? pc : apieces - 1);
        }
        if (TAPS == 9) { // 256 rows: the upper half of the workgroup repeats the lower half's loads and drops them
            const int c = (tid & 255) >> 3, y = tid & 7;
            st.bv[0] = row_fetch<WC>(a.B + ((i64)im * a.Nc + n0 + c) * HW, y, H, W);
        } else {
            const uint16_t *Bb = a.B + ((i64)im * a.Nc + n0) * HW;
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                const int pc = tid + NT * i;
                st.bv[i] = fetch_item(Bb, pc < bpieces ? pc : bpieces - 1);
            }
        }
    };
    // Item pc goes to its pixel slots.  8x8: a piece is one image row.  7x7: see above.  Otherwise the elements
    // of the piece (elements 8 pc .. 8 pc + 7 of the planes laid end to end) are scattered one by one: pixel (y, x) of a 3x3 stage to slot
    // 8 y + x (rows as k-fragments, x >= W stays zero), pixel p of a 1x1 stage to slot p.
    auto put_raw = [&](unsigned char *dst, int pc, const u32x4 v) __attribute__((always_inline)) {
        if (AL8) {
            *(u32x4_alias *)(dst + (pc >> 3) * 144 + (pc & 7) * 16) = v;
            return;
        }
        if (SQ7) {
            const int plane = pc / 7, c = pc - 7 * plane;
            const u32x4 fixed = TAPS == 9 ? row_fix<7>(v, c, 7) : c == 6 ? u32x4{v.w >> 16, 0u, 0u, 0u} : v;
            *(u32x4_alias *)(dst + plane * 144 + c * 16) = fixed;
            return;
        }
        if (HC == 7 && WC == 7 && TAPS == 1) {
            // 49-pixel planes laid end to end: the piece starts at pixel px0 of a plane and may run on into the
            // next one, whose pixel 0 stands 144 - 98 bytes further on in LDS than in memory.  (A 7 x 7 plane is 98
            // bytes, so a 16-byte request for 8 pixels of one plane is never aligned, and a misaligned request
            // costs the memory pipeline three aligned ones: aligned pieces, taken apart here, are cheaper.)
            const int f0 = 8 * pc, plane = f0 / 49, px0 = f0 - 49 * plane, j = 49 - px0; // elements e >= j: next plane
            unsigned char *b0 = dst + plane * 144 + px0 * 2, *b1 = b0 + 46;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t word = v[e >> 1];
                *(uint16_t *)((e < j ? b0 : b1) + 2 * e) = (uint16_t)((e & 1) ? (word >> 16) : word);
            }
            return;
        }
        const int e = 8 * pc;
        int plane = e / HW, px = e - plane * HW, y = 0, xx = px;
        if (TAPS == 9) {
            y = px / W;
            xx = px - y * W;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t word = v[j >> 1];
            const uint16_t el = (uint16_t)((j & 1) ? (word >> 16) : (word & 0xffffu));
            *(uint16_t *)(dst + plane * 144 + y * 16 + xx * 2) = el;
            ++xx;
            if (TAPS == 9) {
                if (xx == W) {
                    xx = 0;
                    ++y;
                }
                if (y == H) {
                    y = 0;
                    ++plane;
                }
            } else if (xx == HW) {
                xx = 0;
                ++plane;
            }
        }
    };
    auto stage_to_lds = [&](const Stage &st, int buf) __attribute__((always_inline)) {
        unsigned char *Ad = a_buf(buf), *Bd = b_buf(buf);
#pragma unroll
        for (int i = 0; i < APT; ++i) {
            const int pc = tid + NT * i;
            if (pc < apieces) put_raw(Ad, pc, st.av[i]);
        }
        if (TAPS == 9) {
            const int c = tid >> 3, y = tid & 7;
            if (y < H && tid < 256) {
                const u32x4 r = row_fix<WC>(st.bv[0], y, H);
                // tx = 0 reads x - 1: shift towards higher x, zero enters at x = 0
                const u32x4 s0 = {r.x << 16, (r.y << 16) | (r.x >> 16), (r.z << 16) | (r.y >> 16),
                                  (r.w << 16) | (r.z >> 16)};
                // tx = 2 reads x + 1: shift towards lower x, zero enters at x = 7
                const u32x4 s2 = {(r.x >> 16) | (r.y << 16), (r.y >> 16) | (r.z << 16), (r.z >> 16) | (r.w << 16),
                                  r.w >> 16};
                unsigned char *base = Bd + (c * WG_ROWS + y + 1) * 16; // [tx][channel][row][8]
                *(u32x4_alias *)(base) = s0;
                *(u32x4_alias *)(base + NCH * WG_ROWS * 16) = r;
                *(u32x4_alias *)(base + 2 * NCH * WG_ROWS * 16) = s2;
            }
        } else {
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                const int pc = tid + NT * i;
                if (pc < bpieces) put_raw(Bd, pc, st.bv[i]);
            }
        }
    };
    // k-fragment ks of plane `ch`: pixel slots 16 ks + 8 half .. + 7, that is image rows 2 ks, 2 ks + 1 (3x3)
    // or pixels 16 ks .. 16 ks + 15 (1x1)
    auto raw_frag = [&](const unsigned char *src, int ch, int ks) __attribute__((always_inline)) {
        return *(const u32x4_alias *)(src + ch * 144 + (2 * ks + half) * 16);
    };
    auto multiply = [&](int buf) __attribute__((always_inline)) {
        const unsigned char *As = a_buf(buf), *Bs = b_buf(buf);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int ks = 2 * kh + kk;
            if ((TAPS == 9 ? 2 * ks : 16 * ks) < (TAPS == 9 ? H : HW) && p0 < NPAIR) { // (uniform) pixels and pairs to do
                u32x4 af[MBW], bf[PWN];
#pragma unroll
                for (int b = 0; b < MBW; ++b) af[b] = raw_frag(As, 32 * (mb0 + b) + col, ks);
#pragma unroll
                for (int p = 0; p < PWN; ++p) {
                    const int pair = p0 + p < NPAIR ? p0 + p : NPAIR - 1; // a slot past the end repeats the last pair
                    if (TAPS == 9) {
                        const int ty = pair / 3, tx = pair % 3;
                        bf[p] = *(const u32x4_alias *)(Bs + ((tx * NCH + col) * WG_ROWS + 2 * ks + half + ty) * 16);
                    } else {
                        bf[p] = raw_frag(Bs, 32 * pair + col, ks);
                    }
                }
#pragma unroll
                for (int p = 0; p < PWN; ++p)
#pragma unroll
                    for (int b = 0; b < MBW; ++b)
                        acc[b][p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg_bf(af[b]), wg_bf(bf[p]),
                                                                            acc[b][p], 0, 0, 0);
            }
        }
    };

    if (img0 < img1) { // (uniform; an empty group writes zeros below)
        // st[d] holds the image that is staged next-but-d; buffer (s & 1) holds image img0 + s while it is
        // multiplied and the following image is written into the other buffer.
        Stage st[ND];
#pragma unroll
        for (int d = 0; d < ND; ++d) load_image(st[d], img0 + d);
        __syncthreads(); // the zero fill above
        stage_to_lds(st[0], 0);
        load_image(st[0], img0 + ND);
        __syncthreads();
        for (int img = img0; img < img1; img += ND) {
#pragma unroll
            for (int d = 0; d < ND; ++d) {
                if (img + d < img1) { // (uniform)
                    Stage &nx = st[(d + 1) % ND];
                    if (img + d + 1 < img1) stage_to_lds(nx, (d + 1) & 1);
                    load_image(nx, img + d + 1 + ND);
                    multiply(d & 1);
                    __syncthreads(); // the staged image is complete; the buffer just read may be rewritten
                }
            }
        }
    }

    // The two k halves trade: tiles [0, KEEP) end in kh = 0, the others in kh = 1.
    constexpr int KEEP = C::KEEP, TILES = C::TILES;
    __syncthreads(); // (an empty group arrives here straight from the zero fill)
    {
        u32x4_alias *mine = (u32x4_alias *)lds + (size_t)w * KEEP * 256;
        const u32x4_alias *theirs = (const u32x4_alias *)lds + (size_t)(w ^ 1) * KEEP * 256;
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const int b = t / PWN, p = t % PWN;
            const bool send = (t < KEEP) == (kh == 1);
            if (send) { // (uniform)
                const int slot = t < KEEP ? t : t - KEEP;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    mine[(slot * 4 + q) * 64 + lane] =
                        u32x4{__float_as_uint(acc[b][p][4 * q]), __float_as_uint(acc[b][p][4 * q + 1]),
                              __float_as_uint(acc[b][p][4 * q + 2]), __float_as_uint(acc[b][p][4 * q + 3])};
            }
        }
        __syncthreads();
        float *part = a.partial + (i64)g * TAPS * a.M * a.Nc; // partial[g][tap][m][n]
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const int b = t / PWN, p = t % PWN;
            const bool keep = (t < KEEP) == (kh == 0);
            const int pair = p0 + p;
            if (keep && pair < NPAIR) { // (uniform)
                const int slot = t < KEEP ? t : t - KEEP;
                const int nb = pair / TAPS, tap = pair % TAPS;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const u32x4 o = theirs[(slot * 4 + q) * 64 + lane];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = 4 * q + e;
                        const int m = m_off + 32 * (mb0 + b) + 8 * (v >> 2) + 4 * half + (v & 3);
                        // kh = 0 first: the sum does not depend on which half adds it
                        const float ov = __uint_as_float(o[e]);
                        const float lo = kh == 0 ? acc[b][p][v] : ov, hi = kh == 0 ? ov : acc[b][p][v];
                        part[((i64)tap * a.M + m) * a.Nc + n0 + 32 * nb + col] = lo + hi;
                    }
                }
            }
        }
    }
}

// One launch computes both filter gradients: the first nwg1 workgroups work on problem 1 (taps T1: the
// k x k stage), the others on problem 2 (always a 1x1 stage).  Each problem has its own image grouping.
// MB1 / MB2: 32-row blocks of m one workgroup of problem 1 / 2 takes; a 3x3 stage runs as two workgroups of
// half the rows each (nine taps each): more, shorter workgroups for the same partial-sum traffic, and at rank
// 128 the accumulators of all nine taps and 128 rows would not fit one register file.
template <int T1, int MB1, int MB2, int HC, int WC>
__global__ __launch_bounds__(WG_THREADS, 1) void conv_wgrad_pair_kernel(WgradArgs a1, WgradArgs a2, int nx1, int nx2, int nwg1)
{
    typedef WgCfg<T1, MB1, (T1 == 9 ? 1 : 4), HC, WC> C1;
    typedef WgCfg<1, MB2, 4, HC, WC> C2;
    __shared__ __attribute__((aligned(16))) unsigned char wg_lds[C1::LDS_BYTES > C2::LDS_BYTES ? C1::LDS_BYTES : C2::LDS_BYTES];
    const int b = blockIdx.x;
    if (b < nwg1) {
        const int mh = a1.M / (32 * MB1), rest = b / nx1; // m parts per image group
        conv_wgrad_body<T1, MB1, (T1 == 9 ? 1 : 4), HC, WC>(a1, b % nx1, rest / mh, 32 * MB1 * (rest % mh), wg_lds);
    } else {
        conv_wgrad_body<1, MB2, 4, HC, WC>(a2, (b - nwg1) % nx2, (b - nwg1) / nx2, 0, wg_lds);
    }
}

// out[m * s_m + n * s_n + tap * s_tap] (+)= sum_g partial[g][tap][m][n]; four consecutive n per output
// The blocks past blocks01 add up per-tile column sums instead (a bias gradient): 16 columns per block,
// sixteen threads per column take every sixteenth tile, and their sums are added in a fixed order.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(WgradReduceArgs r0, WgradReduceArgs r1, int blocks0,
                                                            ColsumTilesArgs cs, int blocks01)
{
    if ((int)blockIdx.x >= blocks01) {
        __shared__ float part[16][16];
        const int tc = threadIdx.x & 15, tg = threadIdx.x >> 4;
        const int colm = (blockIdx.x - blocks01) * 16 + tc;
        const float *p = cs.partial + colm;
        float acc = 0.f;
        for (int t = tg; t < cs.tiles; t += 256) { // sixteen loads in flight (tiles past the end repeat the last, unused)
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = p[(i64)min(t + 16 * u, cs.tiles - 1) * cs.cols];
#pragma unroll
            for (int u = 0; u < 16; ++u) acc += t + 16 * u < cs.tiles ? v[u] : 0.f;
        }
        part[tg][tc] = acc;
        __syncthreads();
        if (tg == 0) {
            float sum = 0.f;
#pragma unroll
            for (int u = 0; u < 16; ++u) sum += part[u][tc];
            cs.out[colm] = cs.accumulate ? cs.out[colm] + sum : sum;
        }
        return;
    }
    // 64 outputs of four floats per block; the groups are dealt to four threads per output, which add their
    // share with up to eight loads in flight, and the four sums are added in a fixed order.
    const bool second = (int)blockIdx.x >= blocks0;
    const WgradReduceArgs r = second ? r1 : r0;
    const int q = threadIdx.x >> 6, o = threadIdx.x & 63;
    const i64 count = (i64)r.taps * r.M * r.Nc; // multiple of 4: Nc is a multiple of 32
    const i64 stride4 = count / 4;
    const i64 i4 = (i64)(blockIdx.x - (second ? blocks0 : 0)) * 64 + o;
    const bool live = i4 < stride4;
    const float4 *p = (const float4 *)r.partial + (live ? i4 : stride4 - 1);
    const int per = (r.groups + 3) / 4, gend = min(r.groups, (q + 1) * per);
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    int g = q * per;
    for (; g + 8 <= gend; g += 8) {
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
    if (g < gend) { // the last groups of this share, again all in flight together
        float4 v[7];
#pragma unroll
        for (int k = 0; k < 7; ++k) v[k] = p[(i64)(g + k < gend ? g + k : gend - 1) * stride4];
#pragma unroll
        for (int k = 0; k < 7; ++k) {
            if (g + k < gend) {
                s.x += v[k].x;
                s.y += v[k].y;
                s.z += v[k].z;
                s.w += v[k].w;
            }
        }
    }
    __shared__ float4 shares[4][64];
    shares[q][o] = s;
    __syncthreads();
    if (q != 0 || !live) return;
#pragma unroll
    for (int k = 1; k < 4; ++k) {
        const float4 t = shares[k][o];
        s.x += t.x;
        s.y += t.y;
        s.z += t.z;
        s.w += t.w;
    }
    const i64 i = 4 * i4;
    const int n = (int)(i % r.Nc);
    const i64 t = i / r.Nc;
    const int m = (int)(t % r.M), tap = (int)(t / r.M);
    float *dst = r.out + m * r.s_m + n * r.s_n + tap * r.s_tap;
    float v[4] = {s.x, s.y, s.z, s.w};
    if (r.nscale) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] *= r.nscale[n + e];
    }
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
    (void)which;
    return k == 3 ? 32 : 128;
}

// a1: the k x k stage (k = 3 or 1); a2: the 1x1 stage; either may be skipped by passing partial == NULL.
int launch_conv_wgrad_pair(hipStream_t s, const WgradArgs &a1, int k1, const WgradArgs &a2)
{
    int st = PF_OK;
    if (a1.N_img <= 0) return st;
    const int M = a1.M;
    if ((M != 64 && M != 128) || a2.M != M || (k1 != 1 && k1 != 3)) return PF_ERR_UNSUPPORTED;
    const int mb1 = k1 == 3 ? M / 64 : M / 32; // 32-row blocks per workgroup of problem 1 (3x3: half the rows)
    const int nx1 = a1.partial ? a1.Nc / wgrad_nchunk(M, k1, 1) : 0;
    const int nx2 = a2.partial ? a2.Nc / wgrad_nchunk(M, 1, 2) : 0;
    const int nwg1 = nx1 * a1.groups * (M / (32 * mb1)), nwg2 = nx2 * a2.groups;
    if (nwg1 + nwg2 == 0) return st;
    const dim3 grid(nwg1 + nwg2), block(WG_THREADS);
    const int x1 = nx1 > 0 ? nx1 : 1, x2 = nx2 > 0 ? nx2 : 1;
    const bool sq8 = a1.H == 8 && a1.W == 8, sq7 = a1.H == 7 && a1.W == 7;
#define PF_WGRAD_CASE(T1, MB1, MB2)                                                                                \
    if (k1 * k1 == T1 && mb1 == MB1 && M == 32 * MB2) {                                                            \
        if (sq8) {                                                                                                 \
            PF_LAUNCH(st, "conv_wgrad_pair", (conv_wgrad_pair_kernel<T1, MB1, MB2, 8, 8>), grid, block, s, a1, a2, \
                      x1, x2, nwg1);                                                                               \
        } else if (sq7) {                                                                                          \
            PF_LAUNCH(st, "conv_wgrad_pair", (conv_wgrad_pair_kernel<T1, MB1, MB2, 7, 7>), grid, block, s, a1, a2, \
                      x1, x2, nwg1);                                                                               \
        } else {                                                                                                   \
            PF_LAUNCH(st, "conv_wgrad_pair", (conv_wgrad_pair_kernel<T1, MB1, MB2, 0, 0>), grid, block, s, a1, a2, \
                      x1, x2, nwg1);                                                                               \
        }                                                                                                          \
        return st;                                                                                                 \
    }
    PF_WGRAD_CASE(9, 1, 2)
    PF_WGRAD_CASE(9, 2, 4)
    PF_WGRAD_CASE(1, 2, 2)
    PF_WGRAD_CASE(1, 4, 4)
#undef PF_WGRAD_CASE
    return PF_ERR_UNSUPPORTED;
}

int launch_wgrad_reduce(hipStream_t s, const WgradReduceArgs &r0, const WgradReduceArgs &r1, const ColsumTilesArgs *cs)
{
    int st = PF_OK;
    const i64 c0 = r0.out ? (i64)r0.taps * r0.M * r0.Nc : 0, c1 = r1.out ? (i64)r1.taps * r1.M * r1.Nc : 0;
    const int b0 = (int)((c0 / 4 + 63) / 64), b1 = (int)((c1 / 4 + 63) / 64);
    ColsumTilesArgs c = {};
    if (cs && cs->out && cs->tiles > 0) c = *cs;
    if (c.cols % 16 != 0) return PF_ERR_UNSUPPORTED;
    const int b2 = c.cols / 16;
    if (b0 + b1 + b2 == 0) return st;
    PF_LAUNCH(st, "wgrad_reduce", wgrad_reduce_kernel, dim3(b0 + b1 + b2), dim3(256), s, r0, r1, b0, c, b0 + b1);
    return st;
}

} // namespace pf
