// Fused two-stage convolution chain kernel (see pf_conv_chain.h) and its weight packers.
#include "pf_conv_chain.h"

namespace pf {

constexpr int CH_PIX = 64;           // pixel slots of one image tile
constexpr int CH_PP = 101;           // padded positions (up to 10 x 10) plus one all-zero row
constexpr int CH_SUB = 64;           // channels staged per wavefront at a time
constexpr int CH_XLD = CH_SUB + 8;   // row stride (elements) of the staged input tile: 144 bytes
constexpr int CH_PLD = 64 + 4;        // stride (floats) between the pixels of a partial-sum tile [pixel][64 rows of rho]

typedef uint4 __attribute__((may_alias)) uint4_alias;
typedef uint32_t xvec_t __attribute__((ext_vector_type(4))); // native vector: stays in registers inside an array
typedef xvec_t __attribute__((may_alias)) xvec_alias;

// 16-byte LDS fragment read that may alias the 2-byte stores which filled the tile
__device__ __forceinline__ uint4 lds_read16(const uint16_t *p) { return *(const uint4_alias *)p; }

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v)
{
    union {
        uint4 u;
        bf16x8_t b;
    } c;
    c.u = v;
    return c.b;
}

// HC, WC: image height / width known at compile time (0 = read them from the arguments).
// CL ("channels last", the fully connected layer): the input is a row-major matrix X[rows][C1], one tile =
// 64 consecutive rows standing where the 64 pixels of an image stand; the intermediate and the output are
// row-major too (T[rows][R], Y[rows][C2]), a bias may be added, and both stages are 1x1.
// EP: the epilogue members of the arguments are honoured (a separate instantiation, so that the plain layer does
// not carry their registers).
// SPLIT: workgroups per image (1 or 2).  With 2 (a batch that leaves half the chip empty) both run the whole first
// stage and each takes half of the second stage's output blocks, one block per wavefront step instead of a pair:
// half the second-stage weights per workgroup, which is what bounds a 3x3 second stage.
template <int KS1, int KS2, int R, int HC, int WC, bool CL = false, bool EP = false, int SPLIT = 1>
__global__ __launch_bounds__(256, 1) void conv_chain_kernel(ChainArgs a)
{
    constexpr int NB2 = SPLIT == 2 ? 1 : 2;    // output blocks (32 channels) a wavefront works on at a time
    constexpr int NVW = 4 * SPLIT;             // wavefronts that share an image's second stage
    static_assert(SPLIT == 1 || (!CL && !EP), "the split kernel is built for the plain image mode");
    constexpr int RB = R / 32, R16 = R / 16, T1 = KS1 * KS1, T2 = KS2 * KS2;
    constexpr int TLD = R + 8; // row stride (elements) of the intermediate tile
    constexpr int S2 = T2 * R16;
    // Stage-1 weight fragments are fetched one group of GS1 k-steps ahead of the MFMAs that use them,
    // two fragments per k-step, so the vector-memory pipe sees a steady stream instead of bursts.
    constexpr int GS1 = KS1 == 3 ? (R == 64 ? 9 : 3) : 4; // k-steps per group
    constexpr int GPS = 4 * T1 / GS1;                     // groups per 64-channel staging round
    constexpr int NXV = CH_SUB * CH_PIX / 8 / 64;         // staging items per lane per round (upper bound)
    __shared__ __attribute__((aligned(16))) uint16_t Xs[4][CH_PP * CH_XLD];
    __shared__ __attribute__((aligned(16))) float P[4][64 * CH_PLD];
    __shared__ __attribute__((aligned(16))) uint16_t Ts[CH_PP * TLD];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int n = blockIdx.x;
    const int H = HC ? HC : a.H, W = WC ? WC : a.W, HW = H * W, C1 = a.C1, C2 = a.C2;
    const int Wp1 = KS1 == 3 ? W + 2 : W, Wp2 = KS2 == 3 ? W + 2 : W;
    const int Z1 = KS1 == 3 ? (H + 2) * (W + 2) : HW; // index of the all-zero row
    const int Z2 = KS2 == 3 ? (H + 2) * (W + 2) : HW;
    const int cw = C1 / 4;        // stage-1 channels of this wavefront
    const int nsub = cw / CH_SUB; // staging rounds
    const int ngroups = nsub * GPS;
    uint16_t *xs = &Xs[w][0];

    // One staging item = one pixel x 8 consecutive channels (one 16-byte LDS row segment); a lane owns
    // items lane, lane + 64, ...; neighbouring lanes read neighbouring pixels, so the 2-byte loads coalesce.
    //
    // XT: a 1x1 first stage of an 8 x 8 or 7 x 7 image needs no shifted reads, so the 64 planes of a round stay
    // as they are in memory -- tile row = channel, 64 pixel slots (pitch CH_XLD) -- copied with 16-byte loads
    // in memory order, and the transposing LDS read turns them into MFMA fragments (the pixel-by-pixel gather
    // costs eight 2-byte loads per item on the unit that also carries the weight stream).  A 7 x 7 plane is 98
    // bytes: one unaligned load per group of 8 slots, the last group read from further back so that it stays
    // in the plane.  (Aligned loads of the planes laid end to end, written to their slots with 16-byte LDS
    // stores at 2-byte aligned addresses, were measured: the misaligned LDS stores cost more than the
    // misaligned global loads, 3.8 k against 2.8 k cycles per 64-channel round.)
    constexpr bool XT = !CL && KS1 == 1 && HC == 8 && WC == 8;
    constexpr int XG = 8; // 16-byte items per plane
    // XF: a 1x1 first stage of a 7 x 7 image.  A plane is 98 bytes, so neither the planes nor 8-pixel pieces of them
    // are aligned, and a 16-byte request at a 2-byte aligned address costs the memory pipeline three aligned ones.
    // But 256 consecutive planes are 1568 aligned 16-byte pieces: the workgroup copies them to LDS as they are
    // (two buffers, one barrier per round), and wavefront w multiplies the channels 4 i + w of the block (the
    // packed weights are ordered to match).  Its rows then start 392 bytes apart at 98 w bytes, which is 2 w past a
    // multiple of 8: it reads them from w elements earlier, so that the transposing read gets aligned addresses,
    // and its pixel p stands in slot p + w.  The slots before and after the 49 pixels hold neighbouring planes'
    // pixels; their columns of the product are never looked at, and the partial sums are lined up when the four
    // wavefronts' tiles are added.
    constexpr bool XF = !CL && KS1 == 1 && HC == 7 && WC == 7;
    constexpr int XF_VEC = 256 * 49 / 8;       // 16-byte pieces of a block of 256 planes
    constexpr int XF_ELEMS = 256 * 49 + 16;    // elements of one buffer (the last row is read 11 elements past the block)
    static_assert(!XF || 2 * XF_ELEMS <= 4 * CH_PP * CH_XLD, "two flat buffers fit in the input tiles");
    uint16_t *const xf0 = &Xs[0][0];
    int xf_buf = 0; // buffer the MFMAs read
    xvec_t xv[NXV];
    const int nitem = 8 * HW;
    auto load_x = [&](int sub) __attribute__((always_inline)) {
        if (CL) { // item = (row m, channel octet o): 16 contiguous bytes of X; rows past the end re-read the last row
#pragma unroll
            for (int i = 0; i < NXV; ++i) {
                const int it = lane + 64 * i, m = it >> 3, o = it & 7;
                i64 row = (i64)n * CH_PIX + m;
                row = row < a.rows ? row : a.rows - 1;
                xv[i] = *(const xvec_t *)(a.in + row * C1 + w * cw + sub * CH_SUB + 8 * o);
            }
            return;
        }
        if (XF) { // round `sub` = planes 256 sub .. 256 sub + 255 of the image, piece tid + 256 i to this thread
            const uint16_t *blk = a.in + ((i64)n * C1 + sub * 256) * 49;
#pragma unroll
            for (int i = 0; i < 7; ++i) xv[i] = *(const xvec_t *)(blk + 8 * min(tid + 256 * i, XF_VEC - 1));
            return;
        }
        const uint16_t *src = a.in + ((i64)n * C1 + w * cw + sub * CH_SUB) * HW;
        if (XT) {
#pragma unroll
            for (int i = 0; i < NXV; ++i) {
                const int it = min(lane + 64 * i, CH_SUB * XG - 1), ch = it / XG, j = it - ch * XG;
                xv[i] = *(const xvec_t *)(src + ch * 64 + 8 * j);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < NXV; ++i) {
            const int it = lane + 64 * i;
            uint32_t e[8];
            if (it < nitem) {
                const int o = it / HW, p = it - o * HW;
                const uint16_t *q = src + (8 * o) * HW + p;
#pragma unroll
                for (int k = 0; k < 8; ++k) e[k] = q[k * HW];
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) e[k] = 0;
            }
            xv[i] = xvec_t{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
        }
    };
    auto store_x = [&]() __attribute__((always_inline)) {
        if (CL) {
#pragma unroll
            for (int i = 0; i < NXV; ++i) {
                const int it = lane + 64 * i, m = it >> 3, o = it & 7;
                *(xvec_alias *)&xs[m * CH_XLD + 8 * o] = xv[i];
            }
            return;
        }
        if (XF) { // into the buffer that is not being read
            uint16_t *dstb = xf0 + (xf_buf ^ 1) * XF_ELEMS;
#pragma unroll
            for (int i = 0; i < 7; ++i) {
                const int vi = tid + 256 * i;
                if (vi < XF_VEC) *(xvec_alias *)&dstb[8 * vi] = xv[i];
            }
            return;
        }
        if (XT) {
#pragma unroll
            for (int i = 0; i < NXV; ++i) {
                const int it = lane + 64 * i, ch = it / XG, j = it - ch * XG;
                if (it < CH_SUB * XG) *(xvec_alias *)&xs[ch * CH_XLD + 8 * j] = xv[i];
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < NXV; ++i) {
            const int it = lane + 64 * i;
            if (it < nitem) {
                const int o = it / HW, p = it - o * HW;
                const int y = p / W, x = p - y * W;
                const int pos = KS1 == 3 ? (y + 1) * Wp1 + x + 1 : p;
                *(xvec_alias *)&xs[pos * CH_XLD + 8 * o] = xv[i];
            }
        }
    };
    const uint4 *w1s = a.W1p + ((i64)(w * cw / 16) * T1 * RB) * 64 + lane; // this wavefront's fragment stream
    // Workgroups that share an L2 (every 8th one) start at different groups, so that between them they pull
    // the whole weight stream into that L2 early instead of all missing on the same lines at the same time.
    const int rot1 = nsub > 1 ? (int)((n >> 3) % nsub) * GPS : (int)((n >> 3) % GPS);
    auto grp = [&](int g) __attribute__((always_inline)) { // g-th group in this workgroup's order (clamped)
        const int r = (g < ngroups ? g : ngroups - 1) + rot1;
        return r >= ngroups ? r - ngroups : r;
    };
    // ---- zero the tiles (borders and the spare row stay zero for the whole kernel): first, because these stores need
    // nothing from memory, while the requests below keep the wavefront at the memory pipeline's door for a while ----
    {
        const uint4 z = make_uint4(0, 0, 0, 0);
        uint4_alias *x4 = (uint4_alias *)&Xs[0][0];
        if (!XF) // (the flat copy needs no zeros)
            for (int i = tid; i < 4 * CH_PP * CH_XLD / 8; i += 256) x4[i] = z;
        uint4_alias *t4 = (uint4_alias *)&Ts[0];
        for (int i = tid; i < CH_PP * TLD / 8; i += 256) t4[i] = z;
    }
    uint4 afA[GS1][RB], afB[GS1][RB];
    load_x(grp(0) / GPS);
    {
        const uint4 *src = w1s + (i64)grp(0) * GS1 * RB * 64;
#pragma unroll
        for (int t = 0; t < GS1; ++t)
#pragma unroll
            for (int b = 0; b < RB; ++b) afA[t][b] = src[(t * RB + b) * 64];
    }

    if (!XF) __syncthreads(); // (the flat copy's first round ends with a barrier of its own, and it writes no zeroed tile)

    // top-left padded position of this lane's two pixels (pixel blocks 0 and 1), both stages,
    // as element offsets into the tiles; lanes without a pixel read the all-zero row
    int base1[2], base2[2];
    bool valid[2];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        const int p = 32 * pb + col;
        const int y = p / W, x = p - y * W;
        valid[pb] = p < HW;
        base1[pb] = (valid[pb] ? (KS1 == 3 ? y * Wp1 + x : p) : Z1) * CH_XLD + 8 * half;
        base2[pb] = (valid[pb] ? (KS2 == 3 ? y * Wp2 + x : p) : Z2) * TLD + 8 * half;
    }

    // ------------------------------- stage 1 -------------------------------
    f32x16_t acc[RB][2];
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][pb][v] = 0.f;

    // input fragment offset (elements) of k-step t of group g, before the lane's base
    auto xoff = [&](int gi, int t) __attribute__((always_inline)) {
        if (KS1 == 3 && GS1 == 9) return ((t / 3) * Wp1 + (t % 3)) * CH_XLD + 16 * gi;
        if (KS1 == 3) return ((gi % 3) * Wp1 + t) * CH_XLD + 16 * (gi / 3);
        return 16 * t;
    };
    // input fragment of pixel block pb: 8 consecutive channels of this lane's pixel
    auto xfrag = [&](int pb, int gi, int t) __attribute__((always_inline)) {
        if (XF) {
            union {
                bf16x8_t b;
                uint4 u;
            } c;
            c.b = lds_frag_tr(xf0 + xf_buf * XF_ELEMS + 48 * w, 4 * 49, 16 * t, 32 * pb, lane);
            return c.u;
        }
        if (XT) { // (slots past the image hold zeros)
            union {
                bf16x8_t b;
                uint4 u;
            } c;
            c.b = lds_frag_tr(xs, CH_XLD, 16 * t, 32 * pb, lane);
            return c.u;
        }
        return lds_read16(&xs[base1[pb] + (valid[pb] ? xoff(gi, t) : 0)]);
    };
    // multiply group g (fragments in cur) while fetching the fragments of group gn into nxt
    auto run_group = [&](const uint4(&cur)[GS1][RB], uint4(&nxt)[GS1][RB], int g, int gn) __attribute__((always_inline)) {
        const int gi = g % GPS;
        const uint4 *src = w1s + (i64)gn * GS1 * RB * 64;
        uint4 bc[2], bn[2];
#pragma unroll
        for (int pb = 0; pb < 2; ++pb) bc[pb] = xfrag(pb, gi, 0);
#pragma unroll
        for (int t = 0; t < GS1; ++t) {
#pragma unroll
            for (int b = 0; b < RB; ++b) nxt[t][b] = src[(t * RB + b) * 64];
            if (t + 1 < GS1) {
#pragma unroll
                for (int pb = 0; pb < 2; ++pb) bn[pb] = xfrag(pb, gi, t + 1);
            }
#pragma unroll
            for (int b = 0; b < RB; ++b)
#pragma unroll
                for (int pb = 0; pb < 2; ++pb)
                    acc[b][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(cur[t][b]), as_bf16x8(bc[pb]), acc[b][pb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int pb = 0; pb < 2; ++pb) bc[pb] = bn[pb];
        }
    };
    // after the g-th group: if it closed a staging round, bring in the next 64 channels (rounds are
    // entered at their first group because the rotation is a whole number of rounds when nsub > 1)
    auto next_round = [&](int g) __attribute__((always_inline)) {
        if ((g + 1) % GPS == 0 && g + 1 < ngroups) {
            // (the tile belongs to this wavefront alone, and a wavefront's LDS accesses are performed in the
            // order it issues them: no workgroup barrier, the four wavefronts drift apart freely in stage 1)
            __builtin_amdgcn_wave_barrier();
            store_x();
            if (g + 1 + GPS < ngroups) load_x(grp(g + 1 + GPS) / GPS);
            if (XF) { // the buffers are shared: the round just written becomes the one that is read
                __syncthreads();
                xf_buf ^= 1;
            }
            __builtin_amdgcn_wave_barrier();
        }
    };

    if (XF) xf_buf = 1; // (store_x fills the other buffer: the first round goes to buffer 0)
    store_x();
    if (nsub > 1) load_x(grp(GPS) / GPS);
    if (XF) {
        __syncthreads();
        xf_buf = 0;
    }
    // (otherwise the tile is this wavefront's own: no workgroup barrier)
    __builtin_amdgcn_wave_barrier();
    for (int g = 0; g < ngroups; g += 2) {
        run_group(afA, afB, grp(g), grp(g + 1));
        next_round(g);
        if (g + 1 < ngroups) {
            run_group(afB, afA, grp(g + 1), grp(g + 2));
            next_round(g + 1);
        }
    }

    // stage-2 weight fragments, one tap (R16 k-steps, two 32-channel output blocks) per group;
    // the first group is requested now so that it arrives during the partial-sum exchange
    const int nb2 = C2 / 32;
    const int vw = SPLIT == 2 ? w + 4 * (int)blockIdx.y : w; // this wavefront among those of the image
    const int npair = (nb2 / NB2 + NVW - 1 - vw) / NVW; // output-block pairs (blocks) of this wavefront: NB2 vw, NB2 (vw + NVW), ...
    const int ngroups2 = npair * T2;
    const int rot2 = (int)((n >> 3) % T2);
    // ... and the workgroups that share an L2 start at different pairs, so that they do not all ask it for the same
    // lines of the second-stage weights at the same time
    const int rotp = npair > 0 ? (int)((n >> 3) % npair) : 0;
    auto pair_of = [&](int q) __attribute__((always_inline)) { // which of this wavefront's pairs group q works on
        const int j = q / T2 + rotp;
        return j >= npair ? j - npair : j;
    };
    auto tap_of = [&](int q) __attribute__((always_inline)) { // taps of a pair are visited in a rotated order
        const int t = q % T2 + rot2;
        return t >= T2 ? t - T2 : t;
    };
    // A 1x1 second stage can read its weights where they are ([C2][R], rows are k-contiguous already):
    // fragment (block, k) of a lane is the 16 bytes at row 32 block + lane % 32, column 16 k + 8 (lane / 32).
    const bool w2nat = KS2 == 1 && a.W2nat != nullptr;
    const i64 w2bb = w2nat ? 4 * R : (i64)S2 * 64, w2k = w2nat ? 2 : 64; // strides in 16-byte units
    auto w2src = [&](int q) __attribute__((always_inline)) {
        const int qq = q < ngroups2 ? q : ngroups2 - 1;
        const int ob = NB2 * (vw + NVW * pair_of(qq)), tap = tap_of(qq);
        if (w2nat) return (const uint4 *)(a.W2nat + ((i64)(32 * ob + col) * R + 8 * half));
        return a.W2p + ((i64)ob * S2 + tap * R16) * 64 + lane;
    };
    uint4 bwA[NB2][R16], bwB[NB2][R16];
    // The first group's fragments are requested a few at a time between the phases of the exchange below (pieces
    // [lo, hi) of the NB2 * R16): issued in one go they keep the wavefront at the memory pipeline's door for over a
    // thousand cycles in which the exchange, which only needs LDS, could run.
    constexpr int W2N = NB2 * R16, W2SLOTS = 3 * (R / 64), W2PER = (W2N + W2SLOTS - 1) / W2SLOTS;
    const uint4 *const w2first = w2src(0);
    auto w2_request = [&](int slot) __attribute__((always_inline)) {
        if (ngroups2 > 0) { // (uniform)
#pragma unroll
            for (int i = slot * W2PER; i < (slot + 1) * W2PER && i < W2N; ++i)
                bwA[i / R16][i % R16] = w2first[(i / R16) * w2bb + (i % R16) * w2k];
        }
    };

    // ---------------- sum the four partial tiles, 64 rows of rho at a time ----------------
#pragma unroll
    for (int rh = 0; rh < R / 64; ++rh) {
        if (rh > 0) __syncthreads();
        // a lane holds four consecutive rows of rho per accumulator quad: the tile is pixel-major, so they leave
        // as one 16-byte store (and come back below as 16-byte loads): a quarter of the LDS instructions
        float *pw = &P[w][col * CH_PLD + 4 * half];
#pragma unroll
        for (int bb = 0; bb < 2; ++bb)
#pragma unroll
            for (int pb = 0; pb < 2; ++pb)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *(float4 *)&pw[32 * pb * CH_PLD + 32 * bb + 8 * q] =
                        make_float4(acc[2 * rh + bb][pb][4 * q], acc[2 * rh + bb][pb][4 * q + 1],
                                    acc[2 * rh + bb][pb][4 * q + 2], acc[2 * rh + bb][pb][4 * q + 3]);
        w2_request(3 * rh);
        __syncthreads();
        const int pix = tid & 63;
        const int py = pix / W, px = pix - py * W;
        const int ppos = KS2 == 3 ? (py + 1) * Wp2 + px + 1 : pix;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int r0 = 8 * ((tid >> 6) + 4 * it);
            float f[8];
#pragma unroll
            for (int h4 = 0; h4 < 2; ++h4) {
                // (XF: wavefront k holds pixel p in slot p + k)
                const int idx = pix * CH_PLD + r0 + 4 * h4, sh = XF ? (pix < 61 ? CH_PLD : 0) : 0;
                const float4 p0 = *(const float4 *)&P[0][idx], p1 = *(const float4 *)&P[1][idx + sh];
                const float4 p2 = *(const float4 *)&P[2][idx + 2 * sh], p3 = *(const float4 *)&P[3][idx + 3 * sh];
                f[4 * h4 + 0] = (p0.x + p1.x) + (p2.x + p3.x);
                f[4 * h4 + 1] = (p0.y + p1.y) + (p2.y + p3.y);
                f[4 * h4 + 2] = (p0.z + p1.z) + (p2.z + p3.z);
                f[4 * h4 + 3] = (p0.w + p1.w) + (p2.w + p3.w);
            }
            if (pix < HW) {
                const uint4 pk = make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                                            pack_bf16x2(f[6], f[7]));
                *(uint4_alias *)&Ts[ppos * TLD + 64 * rh + r0] = pk;
                if (a.mid_save && CL) {
                    const i64 row = (i64)n * CH_PIX + pix;
                    if (row < a.rows) *(uint4 *)(a.mid_save + row * R + 64 * rh + r0) = pk;
                } else if (a.mid_save && (SPLIT == 1 || blockIdx.y == 0)) {
                    // The copy kept for the backward pass is [R][HW]: these 8 rows of it are HW 16-byte pieces in a
                    // row.  They are put together in this wavefront's idle input tile and leave below as aligned
                    // 16-byte stores (2-byte stores from here cost the memory pipeline sixteen times as many
                    // instructions, and the barrier below would wait for them).
                    uint16_t *ms = xs + (2 * rh + it) * 8 * CH_PIX + pix;
                    const uint32_t d[4] = {pk.x, pk.y, pk.z, pk.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e) ms[e * HW] = (uint16_t)(d[e >> 1] >> (16 * (e & 1)));
                }
            }
            w2_request(3 * rh + 1 + it);
        }
    }
    __syncthreads();
    if (a.mid_save && !CL && (SPLIT == 1 || blockIdx.y == 0)) { // rows 64 rh + 8 (w + 4 it) .. + 7 of the intermediate, from this wavefront's tile
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int ck = 0; ck < R / 32; ++ck) { // chunk ck = 2 rh + it
            const int r0 = 64 * (ck >> 1) + 8 * (w + 4 * (ck & 1));
            uint4 *dst = (uint4 *)(a.mid_save + ((i64)n * R + r0) * HW);
            if (lane < HW) dst[lane] = *(const uint4_alias *)&xs[ck * 8 * CH_PIX + 8 * lane];
        }
    }

    // ------------------------------- stage 2 -------------------------------
    f32x16_t acc2[NB2][2];
#pragma unroll
    for (int bb = 0; bb < NB2; ++bb)
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc2[bb][pb][v] = 0.f;

    // epilogue operands of the output-block pair in work (16-byte pieces of the pair's 64 x HW block), requested
    // when the pair starts so that they have arrived when it is stored
    constexpr int NOV = CH_PIX * CH_PIX / 8 / 64;
    uint4 epa[NOV], epm[NOV];
    const bool ep_any = EP && !CL && (a.ep_add || a.ep_mask || a.ep_relu);
    auto run_group2 = [&](const uint4(&cur)[NB2][R16], uint4(&nxt)[NB2][R16], int q) __attribute__((always_inline)) {
        const int tap = tap_of(q);
        if (EP && !CL && q % T2 == 0 && (a.ep_add || a.ep_mask)) {
            const i64 blk = ((i64)n * C2 + 32 * NB2 * (vw + NVW * pair_of(q))) * HW;
#pragma unroll
            for (int i = 0; i < NOV; ++i) {
                const int vi = min(lane + 64 * i, 32 * NB2 * HW / 8 - 1);
                if (a.ep_add) epa[i] = ((const uint4 *)(a.ep_add + blk))[vi];
                if (a.ep_mask) epm[i] = ((const uint4 *)(a.ep_mask + blk))[vi];
            }
        }
        const int toff = (KS2 == 3 ? (tap / 3) * Wp2 + (tap % 3) : 0) * TLD;
        const uint4 *src = w2src(q + 1);
        uint4 bc[2], bn[2];
#pragma unroll
        for (int pb = 0; pb < 2; ++pb) bc[pb] = lds_read16(&Ts[base2[pb] + (valid[pb] ? toff : 0)]);
#pragma unroll
        for (int k = 0; k < R16; ++k) {
#pragma unroll
            for (int bb = 0; bb < NB2; ++bb) nxt[bb][k] = src[bb * w2bb + k * w2k];
            if (k + 1 < R16) {
#pragma unroll
                for (int pb = 0; pb < 2; ++pb) bn[pb] = lds_read16(&Ts[base2[pb] + (valid[pb] ? toff : 0) + 16 * (k + 1)]);
            }
#pragma unroll
            for (int pb = 0; pb < 2; ++pb) {
#pragma unroll
                for (int bb = 0; bb < NB2; ++bb)
                    acc2[bb][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(cur[bb][k]), as_bf16x8(bc[pb]), acc2[bb][pb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int pb = 0; pb < 2; ++pb) bc[pb] = bn[pb];
        }
        if (q % T2 == T2 - 1) { // this output-block pair is complete: store it and start the next
            // The 64 output channels x HW pixels of the pair are one contiguous block of `out`.  Round to
            // bf16 into this wavefront's (now idle) input tile laid out exactly like that block, then
            // copy it out with 16-byte stores.
            const int ob = NB2 * (vw + NVW * pair_of(q));
            if (CL) {
                // Row-major output: a lane holds 4 consecutive output channels of one row per accumulator
                // quad.  Stage the 64 rows x 64 channels of the pair in the idle input tile ([row][channel],
                // rows 144 bytes apart), then write 16 bytes per lane: 8 lanes cover one row's 128 bytes.
                const uint16_t *bias = (const uint16_t *)a.bias;
#pragma unroll
                for (int bb = 0; bb < 2; ++bb)
#pragma unroll
                    for (int pb = 0; pb < 2; ++pb) {
#pragma unroll
                        for (int v4 = 0; v4 < 4; ++v4) {
                            const int oc = 32 * bb + 8 * v4 + 4 * half; // channel within the pair's 64
                            float f[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) f[e] = acc2[bb][pb][4 * v4 + e];
                            if (bias) {
                                const uint2 bv = *(const uint2 *)(bias + 32 * ob + oc);
                                f[0] += bf16_bits_to_float((uint16_t)bv.x);
                                f[1] += bf16_bits_to_float((uint16_t)(bv.x >> 16));
                                f[2] += bf16_bits_to_float((uint16_t)bv.y);
                                f[3] += bf16_bits_to_float((uint16_t)(bv.y >> 16));
                            }
                            uint2 pk2;
                            pk2.x = pack_bf16x2(f[0], f[1]);
                            pk2.y = pack_bf16x2(f[2], f[3]);
                            *(uint2 __attribute__((may_alias)) *)&xs[(32 * pb + col) * CH_XLD + oc] = pk2;
                        }
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc2[bb][pb][v] = 0.f;
                    }
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int it = lane + 64 * i, m = it >> 3, o8 = it & 7;
                    const i64 row = (i64)n * CH_PIX + m;
                    if (row < a.rows)
                        *(uint4 *)(a.out + row * C2 + 32 * ob + 8 * o8) = *(const uint4_alias *)&xs[m * CH_XLD + 8 * o8];
                }
                return;
            }
            uint16_t *ys = xs + (4 * half) * HW + col;
            if (EP && (a.ep_scale || a.ep_shift)) { // per output channel, in float, before the one rounding to bf16
#pragma unroll
                for (int bb = 0; bb < NB2; ++bb)
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        const int ch = 32 * ob + 32 * bb + 8 * qd + 4 * half; // four consecutive channels
                        const float4 sc = a.ep_scale ? *(const float4 *)(a.ep_scale + ch) : make_float4(1.f, 1.f, 1.f, 1.f);
                        const float4 sh = a.ep_shift ? *(const float4 *)(a.ep_shift + ch) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                        for (int pb = 0; pb < 2; ++pb) {
                            acc2[bb][pb][4 * qd + 0] = acc2[bb][pb][4 * qd + 0] * sc.x + sh.x;
                            acc2[bb][pb][4 * qd + 1] = acc2[bb][pb][4 * qd + 1] * sc.y + sh.y;
                            acc2[bb][pb][4 * qd + 2] = acc2[bb][pb][4 * qd + 2] * sc.z + sh.z;
                            acc2[bb][pb][4 * qd + 3] = acc2[bb][pb][4 * qd + 3] * sc.w + sh.w;
                        }
                    }
            }
#pragma unroll
            for (int bb = 0; bb < NB2; ++bb)
#pragma unroll
                for (int pb = 0; pb < 2; ++pb) {
                    if (32 * pb + col < HW) {
#pragma unroll
                        for (int v = 0; v < 16; v += 2) {
                            const uint32_t pk = pack_bf16x2(acc2[bb][pb][v], acc2[bb][pb][v + 1]);
                            ys[(32 * bb + 8 * (v >> 2) + (v & 3)) * HW + 32 * pb] = (uint16_t)pk;
                            ys[(32 * bb + 8 * (v >> 2) + (v & 3) + 1) * HW + 32 * pb] = (uint16_t)(pk >> 16);
                        }
                    }
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc2[bb][pb][v] = 0.f;
                }
            uint4 *dst = (uint4 *)(a.out + ((i64)n * C2 + 32 * ob) * HW);
            const int nv = 32 * NB2 * HW / 8;
#pragma unroll
            for (int i = 0; i < CH_PIX * CH_PIX / 8 / 64; ++i) {
                const int vi = lane + 64 * i;
                if (vi < nv) {
                    uint4 y = *(const uint4_alias *)&xs[8 * vi];
                    if (EP && ep_any) { // (uniform) residual / skip gradient, activation, mask: on the block as it leaves
                        uint32_t yw[4] = {y.x, y.y, y.z, y.w};
                        const uint32_t aw[4] = {epa[i].x, epa[i].y, epa[i].z, epa[i].w};
                        const uint32_t mw[4] = {epm[i].x, epm[i].y, epm[i].z, epm[i].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float lo = bf16_bits_to_float((uint16_t)yw[e]), hi = bf16_bits_to_float((uint16_t)(yw[e] >> 16));
                            if (a.ep_add) {
                                lo += bf16_bits_to_float((uint16_t)aw[e]);
                                hi += bf16_bits_to_float((uint16_t)(aw[e] >> 16));
                            }
                            if (a.ep_relu) {
                                lo = fmaxf(lo, 0.f);
                                hi = fmaxf(hi, 0.f);
                            }
                            if (a.ep_mask) {
                                lo = bf16_bits_to_float((uint16_t)mw[e]) > 0.f ? lo : 0.f;
                                hi = bf16_bits_to_float((uint16_t)(mw[e] >> 16)) > 0.f ? hi : 0.f;
                            }
                            yw[e] = pack_bf16x2(lo, hi);
                        }
                        y = make_uint4(yw[0], yw[1], yw[2], yw[3]);
                    }
                    dst[vi] = y;
                }
            }
        }
    };
    for (int q = 0; q < ngroups2; q += 2) {
        run_group2(bwA, bwB, q);
        if (q + 1 < ngroups2) run_group2(bwB, bwA, q + 1);
    }
}

// ------------------------------------------------------------------ packers
__device__ __forceinline__ void pack_w1_item(const PackW1 &p, int g)
{
    // one 16-byte fragment slot: ((s * RB + b) * 64 + lane)
    const int lane = g & 63, fb = g >> 6, b = fb % p.RB, s = fb / p.RB;
    const int rho = 32 * b + (lane & 31), tap = s % p.T;
    int c0 = 16 * (s / p.T) + 8 * (lane >> 5), cs = 1; // first channel of the slot and the step between its channels
    if (p.il_cw) { // k-step S of wavefront w = S / (cw / 16): channels 256 sub + 4 (16 t + 8 (lane / 32) + i) + w
        const int S = s / p.T, per = p.il_cw / 16, wv = S / per, rem = S - wv * per;
        c0 = 256 * (rem >> 2) + 4 * (16 * (rem & 3) + 8 * (lane >> 5)) + wv;
        cs = 4;
    }
    uint32_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = p.src[rho * p.s_rho + (c0 + cs * i) * p.s_c + tap * p.s_tap];
    if (p.cscale) {
#pragma unroll
        for (int i = 0; i < 8; ++i) e[i] = float_to_bf16_bits(bf16_bits_to_float((uint16_t)e[i]) * p.cscale[c0 + cs * i]);
    }
    p.dst[g] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
}

__device__ __forceinline__ void pack_w2_item(const PackW2 &p, int g)
{
    // ((ob * S2 + s2) * 64 + lane)
    const int lane = g & 63, fb = g >> 6, s2 = fb % p.S2, ob = fb / p.S2;
    const int o = 32 * ob + (lane & 31), tap = s2 / p.R16, rho0 = 16 * (s2 % p.R16) + 8 * (lane >> 5);
    uint32_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = p.src[p.base + o * p.s_o + (rho0 + i) * p.s_rho + tap * p.s_tap];
    p.dst[g] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
}

// All weight sets of one call in a single launch (any count may be zero).
__global__ __launch_bounds__(256) void pack_chain_kernel(PackW1 p1, PackW2 p2, PackW1 p3, PackW2 p4)
{
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g < p1.n)
        pack_w1_item(p1, g);
    else if (g - p1.n < p2.n)
        pack_w2_item(p2, g - p1.n);
    else if (g - p1.n - p2.n < p3.n)
        pack_w1_item(p3, g - p1.n - p2.n);
    else if (g - p1.n - p2.n - p3.n < p4.n)
        pack_w2_item(p4, g - p1.n - p2.n - p3.n);
}

bool chain_supported(int C1, int C2, int R, int H, int W, int k, int stride, int pad)
{
    if (stride != 1) return false;
    if (!((k == 3 && pad == 1) || (k == 1 && pad == 0))) return false;
    if (H * W > CH_PIX || (H + 2) * (W + 2) > CH_PP - 1) return false;
    if (R != 64 && R != 128) return false;
    if (C1 % 256 || C2 % 256) return false; // both directions of the chain split channels 4 x 64
    return true;
}

size_t chain_w1_elems(int C1, int R, int k) { return (size_t)k * k * C1 * R; }
size_t chain_w2_elems(int C2, int R, int k) { return (size_t)k * k * C2 * R; }

bool chain_w1_interleaved(int k, int H, int W) { return k == 1 && H == 7 && W == 7; }

PackW1 make_pack_w1(const uint16_t *src, uint4 *dst, int C1, int R, int k, i64 s_rho, i64 s_c, i64 s_tap, int H, int W)
{
    PackW1 p;
    p.src = src;
    p.dst = dst;
    p.T = k * k;
    p.RB = R / 32;
    p.n = src ? p.T * (C1 / 16) * p.RB * 64 : 0;
    p.s_rho = s_rho;
    p.s_c = s_c;
    p.s_tap = s_tap;
    p.cscale = nullptr;
    p.il_cw = chain_w1_interleaved(k, H, W) ? C1 / 4 : 0;
    return p;
}

PackW2 make_pack_w2(const uint16_t *src, uint4 *dst, int C2, int R, int k, i64 base, i64 s_o, i64 s_rho, i64 s_tap)
{
    PackW2 p;
    p.src = src;
    p.dst = dst;
    p.R16 = R / 16;
    p.S2 = k * k * p.R16;
    p.n = src ? (C2 / 32) * p.S2 * 64 : 0;
    p.base = base;
    p.s_o = s_o;
    p.s_rho = s_rho;
    p.s_tap = s_tap;
    return p;
}

int launch_pack_chain(hipStream_t s, const PackW1 &p1, const PackW2 &p2, const PackW1 &p3, const PackW2 &p4)
{
    int st = PF_OK;
    const int n = p1.n + p2.n + p3.n + p4.n;
    if (n <= 0) return st;
    PF_LAUNCH(st, "pack_chain", pack_chain_kernel, dim3((n + 255) / 256), dim3(256), s, p1, p2, p3, p4);
    return st;
}

int launch_linear_chain(hipStream_t s, const char *name, const ChainArgs &a, int R)
{
    int st = PF_OK;
    if (a.rows <= 0) return st;
    const dim3 grid((unsigned)((a.rows + CH_PIX - 1) / CH_PIX)), block(256);
    if (R == 64) {
        PF_LAUNCH(st, name, (conv_chain_kernel<1, 1, 64, 8, 8, true>), grid, block, s, a);
    } else if (R == 128) {
        PF_LAUNCH(st, name, (conv_chain_kernel<1, 1, 128, 8, 8, true>), grid, block, s, a);
    } else {
        st = PF_ERR_UNSUPPORTED;
    }
    return st;
}

bool linear_chain_supported(i64 n_in, i64 n_out, i64 r)
{
    return (r == 64 || r == 128) && n_in % 256 == 0 && n_out % 256 == 0;
}

int launch_conv_chain(hipStream_t s, const char *name, const ChainArgs &a, int N, int k1, int k2, int R)
{
    int st = PF_OK;
    if (N <= 0) return st;
    const dim3 grid(N), block(256);
    const int hw = (a.H == 8 && a.W == 8) ? 8 : (a.H == 7 && a.W == 7) ? 7 : 0;
    const bool ep = a.ep_scale || a.ep_shift || a.ep_add || a.ep_mask || a.ep_relu;
    // a batch that fills at most half the chip: two workgroups per image where the second stage is the long one
    if (!ep && k1 == 1 && k2 == 3 && hw == 8 && 2 * N <= 256 && a.C2 % 64 == 0) {
        const dim3 grid2(N, 2);
        if (R == 64) {
            PF_LAUNCH(st, name, (conv_chain_kernel<1, 3, 64, 8, 8, false, false, 2>), grid2, block, s, a);
            return st;
        }
        if (R == 128) {
            PF_LAUNCH(st, name, (conv_chain_kernel<1, 3, 128, 8, 8, false, false, 2>), grid2, block, s, a);
            return st;
        }
    }
#define PF_CHAIN_CASE(K1, K2, RR)                                                                    \
    if (k1 == K1 && k2 == K2 && R == RR) {                                                           \
        if (hw == 8 && ep) {                                                                         \
            PF_LAUNCH(st, name, (conv_chain_kernel<K1, K2, RR, 8, 8, false, true>), grid, block, s, a); \
        } else if (hw == 7 && ep) {                                                                  \
            PF_LAUNCH(st, name, (conv_chain_kernel<K1, K2, RR, 7, 7, false, true>), grid, block, s, a); \
        } else if (ep) {                                                                             \
            PF_LAUNCH(st, name, (conv_chain_kernel<K1, K2, RR, 0, 0, false, true>), grid, block, s, a); \
        } else if (hw == 8) {                                                                        \
            PF_LAUNCH(st, name, (conv_chain_kernel<K1, K2, RR, 8, 8>), grid, block, s, a);           \
        } else if (hw == 7) {                                                                        \
            PF_LAUNCH(st, name, (conv_chain_kernel<K1, K2, RR, 7, 7>), grid, block, s, a);           \
        } else {                                                                                     \
            PF_LAUNCH(st, name, (conv_chain_kernel<K1, K2, RR, 0, 0>), grid, block, s, a);           \
        }                                                                                            \
        return st;                                                                                   \
    }
    PF_CHAIN_CASE(3, 1, 64)
    PF_CHAIN_CASE(1, 3, 64)
    PF_CHAIN_CASE(1, 1, 64)
    PF_CHAIN_CASE(3, 1, 128)
    PF_CHAIN_CASE(1, 3, 128)
    PF_CHAIN_CASE(1, 1, 128)
#undef PF_CHAIN_CASE
    return PF_ERR_UNSUPPORTED;
}

} // namespace pf
