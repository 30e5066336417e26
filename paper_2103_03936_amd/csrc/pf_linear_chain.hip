// Fused fully connected low-rank layer: see pf_linear_chain.h.
//
// Workgroup = 4 wavefronts, 32 rows.
//   stage 1: wavefront w owns rho block w (32 of the 128 rank channels) over the whole contraction, which is
//            cut into chunks of 128.  A chunk of the input rows [32][128] and of W1 [128][128] is copied to
//            LDS (16-byte loads, register rings 4 and 2 chunks deep so that HBM and L2 latency are covered,
//            two LDS buffers, one barrier per chunk).  Per 16-deep k-step: one 16-byte LDS read for the row
//            fragment, two transposing reads for the W1 fragment, one MFMA.
//   stage 2: the 32 x 128 intermediate goes to LDS in bf16 and every wavefront keeps its 8 fragments in
//            registers; wavefront w owns a quarter of the output blocks, two at a time, W2 fragments are
//            16-byte global loads prefetched one pair ahead.  The output pair is turned row-major through a
//            per-wavefront LDS patch and leaves as 16-byte stores.
#include "pf_linear_chain.h"

#include <type_traits>

namespace pf {

// native vectors (plain SSA values for the compiler, unlike the uint4 struct)
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef u32x4_t __attribute__((may_alias)) uint4_alias;
typedef u32x2_t __attribute__((may_alias)) uint2_alias;

constexpr int LC_R = 128;          // rank
constexpr int LC_KC = 128;         // contraction chunk of stage 1
constexpr int LC_XP = LC_KC + 8;   // LDS pitch (elements) of the row chunk: 272 bytes
constexpr int LC_VP = LC_R + 16;   // of the W1 chunk: 288 bytes (32 mod 128, what the transposing read likes)
constexpr int LC_TP = LC_R + 8;    // of the intermediate
constexpr int LC_YP = 64 + 8;      // of the output patch (two 32-wide blocks)

__device__ __forceinline__ bf16x8_t lc_as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }

// NP: pairs of output blocks per wavefront (C2 / 256) when it is one of 1, 2, 4, 8 -- then stage 2 is fully
// unrolled and its W2 fragments are fetched two pairs ahead, the first two during stage 1; NP == 0: any C2.
// MODE 0: one layer.  MODE 1: the groups of LinChainArgs run one after the other in the same workgroup (same
// rows), each with its own output.  MODE 2: the same, but the groups' stage-2 products are summed into one output.
// EP: the epilogue members of the arguments are honoured (MODE 0 only; a separate instantiation, so that the plain
// layer does not carry their registers).
template <int NP, int MODE = 0, bool EP = false>
__global__ __launch_bounds__(256, 1) void linear_chain2_kernel(LinChainArgs args)
{
    __shared__ __attribute__((aligned(16))) uint16_t Xs[2][LC_ROWS * LC_XP];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[2][LC_KC * LC_VP];
    __shared__ __attribute__((aligned(16))) uint16_t Ts[LC_ROWS * LC_TP];
    __shared__ __attribute__((aligned(16))) uint16_t Ys[4][LC_ROWS * LC_YP];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, col = lane & 31;
    const i64 row0 = (i64)blockIdx.x * LC_ROWS;
    const int C1 = args.C1, C2 = args.C2;
    const int nch = C1 / LC_KC;

    struct XR { // a chunk of the input rows in flight (per thread)
        u32x4_t r[2];
    };
    struct VR { // a chunk of W1 in flight
        u32x4_t r[8];
    };
    struct UR { // W2 fragments of a pair of output blocks, and the bias of this lane's row of each block
        u32x4_t r[2][8];
        uint32_t b[2];
    };

    // ---- copy roles: thread -> (row or k, 16-byte column) of a chunk
    const int cr = tid >> 4, co = tid & 15; // 16 threads per 128-element row; 16 rows per pass

    constexpr bool MULTI = MODE != 0, summing = MODE == 2;
    const int G = MULTI ? args.groups : 1;
    constexpr int NSUM = summing ? NP : 1;
    static_assert(!summing || NP == 1 || NP == 2, "the sums of all output blocks stay in registers");
    f32x16_t ysum[NSUM][2]; // stage-2 sums over the groups (summing only)
#pragma unroll
    for (int i = 0; i < NSUM; ++i)
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int v = 0; v < 16; ++v) ysum[i][bi][v] = 0.f;

    for (int gi = 0; gi < G; ++gi) {
    LinChainArgs a = args;
    if (MULTI) {
        a.in += gi * args.gs_in;
        a.W1 += gi * args.gs_W1;
        a.W2 += gi * args.gs_W2;
        if (a.bias) a.bias += gi * args.gs_bias;
        a.out += gi * args.gs_out;
        if (a.mid_save) a.mid_save += gi * args.gs_mid;
        if (a.colsum) a.colsum += gi * args.gs_colsum;
        if (gi > 0) __syncthreads(); // the LDS tiles of the previous group are free
    }
    const uint16_t *xsrc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        i64 row = row0 + cr + 16 * i;
        if (row > a.rows - 1) row = a.rows - 1; // rows past the end re-read the last one; never stored
        xsrc[i] = a.in + row * C1 + 8 * co;
    }
    const uint16_t *vsrc = a.W1 + (i64)cr * LC_R + 8 * co;

    // Loads are unconditional, so that the compiler can count them exactly when it places the waits:
    // a chunk index past the end re-reads the last chunk, and what it brings is never multiplied.
    // Workgroups walk the chunks (and, in stage 2, the output-block pairs) from different starting points, so
    // that they do not all ask the same L2 channel for the same factor rows at the same moment.  Workgroups
    // are dealt round-robin to the 8 XCDs, each with its own L2: neighbours within an XCD are 8 apart.
    const int rot1 = (blockIdx.x >> 3) % nch;
    auto chunk_of = [&](int c) __attribute__((always_inline)) {
        c = min(c, nch - 1) + rot1;
        return c >= nch ? c - nch : c;
    };
    // (one 16-byte piece at a time, so that the requests can be dealt out between the MFMAs: the memory pipeline
    // takes one such instruction per 16 to 20 cycles from the whole workgroup, and a wavefront that issues a burst
    // of them stands still until the last one has been accepted)
    auto load_x1 = [&](XR &x, int c, int i) __attribute__((always_inline)) {
        x.r[i] = *(const uint4_alias *)(xsrc[i] + chunk_of(c) * LC_KC);
    };
    auto load_v1 = [&](VR &v, int c, int i) __attribute__((always_inline)) {
        v.r[i] = *(const uint4_alias *)(vsrc + ((i64)chunk_of(c) * LC_KC + 16 * i) * LC_R);
    };
    auto load_x = [&](XR &x, int c) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 2; ++i) load_x1(x, c, i);
    };
    auto load_v = [&](VR &v, int c) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) load_v1(v, c, i);
    };

    // ---- stage 2 operands: W2 fragments of a pair of output blocks, straight from global memory
    const int obw = C2 / 128; // output blocks per wavefront
    const int rot2 = (blockIdx.x >> 3) % (obw / 2);
    auto pair_of = [&](int g) __attribute__((always_inline)) {
        g = min(g, obw / 2 - 1) + rot2;
        return g >= obw / 2 ? g - obw / 2 : g;
    };
    // W2 rows as they lie in memory: 16 lanes fetch one 256-byte row, an instruction four rows (a lane per
    // row, which is what the MFMA wants, would touch 64 cache lines per instruction instead of 8)
    auto load_u1 = [&](UR &u, int g, int bi, int j) __attribute__((always_inline)) {
        const uint16_t *p = a.W2 + (i64)(32 * (w * obw + 2 * pair_of(g) + bi) + (lane >> 4)) * LC_R + 8 * (lane & 15);
        u.r[bi][j] = *(const uint4_alias *)(p + (i64)4 * j * LC_R);
    };
    // The bias enters as one more k-step of the second product, [T 1] [W2 b]^T: the lane that holds row o of a block
    // (in the lower half of the wavefront: k = 0..7) carries b[o] at k = 0.  Two small requests per pair instead of
    // vector arithmetic on every output.  (No bias: any readable address; the value is masked to zero.)
    auto load_ub = [&](UR &u, int g, int bi) __attribute__((always_inline)) {
        const uint16_t *p = a.bias ? a.bias + 32 * (w * obw + 2 * pair_of(g) + bi) + col : a.W2;
        const uint32_t v = *p;
        u.b[bi] = (a.bias && half == 0) ? v : 0u;
    };
    auto load_u = [&](UR &u, int g) __attribute__((always_inline)) {
#pragma unroll
        for (int bi = 0; bi < 2; ++bi) {
            load_ub(u, g, bi);
#pragma unroll
            for (int j = 0; j < 8; ++j) load_u1(u, g, bi, j);
        }
    };

    XR x0, x1, x2, x3;
    VR v0, v1;
    UR ur[3];
    // Only what the first two chunks need is requested up front; the rest follows once chunk 0 is in LDS,
    // so that the first MFMA does not wait behind a long queue of requests.
    load_x(x0, 0);
    load_v(v0, 0);
    load_x(x1, 1);
    load_v(v1, 1);

    f32x16_t acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc0[v] = acc1[v] = 0.f;

    auto write_x = [&](const XR &xr, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 2; ++i) *(uint4_alias *)&Xs[buf][(cr + 16 * i) * LC_XP + 8 * co] = xr.r[i];
    };
    auto write_v = [&](const VR &vr, int buf, int i) __attribute__((always_inline)) {
        *(uint4_alias *)&Vs[buf][(cr + 16 * i) * LC_VP + 8 * co] = vr.r[i];
    };
    // Chunk c (already in buffer c & 1) is multiplied while chunk c + 1, which has arrived in the registers xn / vn,
    // is written to the other buffer, one piece per k-step between the MFMAs, and each register is refilled as soon
    // as it has been written (chunks c + 5 / c + 3); the fragments of a k-step are read one k-step ahead.  One
    // barrier closes the chunk: after it the written buffer is complete and the buffer just read may be rewritten.
    // `refill`: whether chunks c + 3 (W1) and c + 5 (rows) are to be requested (std::true_type / std::false_type)
    auto step = [&](XR &xn, VR &vn, int c, auto refill, auto extra) __attribute__((always_inline)) {
        if (c >= nch) return; // uniform
        const int buf = c & 1;
        if (a.colsum) { // column sums of the valid rows of this chunk (bias gradient): 16 rows per thread
            const i64 left = a.rows - row0;
            const int nr = left < LC_ROWS ? (int)left : LC_ROWS;
            const int cc = tid & (LC_KC - 1), hr = tid >> 7;
            uint16_t e[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) e[r] = Xs[buf][(16 * hr + r) * LC_XP + cc];
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) s += 16 * hr + r < nr ? bf16_bits_to_float(e[r]) : 0.f;
            a.colsum[((i64)2 * blockIdx.x + hr) * C1 + chunk_of(c) * LC_KC + cc] = s;
        }
        auto body = [&](auto more) __attribute__((always_inline)) {
            u32x4_t xf[2];
            bf16x8_t vf[2];
            xf[0] = *(const uint4_alias *)&Xs[buf][col * LC_XP + 8 * half];
            vf[0] = lds_frag_tr(&Vs[buf][0], LC_VP, 0, 32 * w, lane);
#pragma unroll
            for (int ks = 0; ks < LC_KC / 16; ++ks) {
                if (ks + 1 < LC_KC / 16) {
                    xf[(ks + 1) & 1] = *(const uint4_alias *)&Xs[buf][col * LC_XP + 16 * (ks + 1) + 8 * half];
                    vf[(ks + 1) & 1] = lds_frag_tr(&Vs[buf][0], LC_VP, 16 * (ks + 1), 32 * w, lane);
                }
                if (decltype(more)::value) {
                    if (ks == 0) write_x(xn, buf ^ 1);
                    write_v(vn, buf ^ 1, ks);
                }
                if (decltype(refill)::value) {
                    if (ks == 1 || ks == 2) load_x1(xn, c + 5, ks - 1);
                    load_v1(vn, c + 3, ks);
                }
                extra(ks);
                if (ks & 1)
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[ks & 1], lc_as_bf16x8(xf[ks & 1]), acc1, 0, 0, 0);
                else
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[ks & 1], lc_as_bf16x8(xf[ks & 1]), acc0, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        if (c + 1 < nch) // uniform
            body(std::true_type{});
        else
            body(std::false_type{});
        __syncthreads();
    };
    auto none = [](int) __attribute__((always_inline)) {};
    auto want_u0 = [&](int ks) __attribute__((always_inline)) { // the stage-2 operands of the first pair ...
        if (ks < 2) load_ub(ur[0], 0, ks);
        load_u1(ur[0], 0, 0, ks);
        load_u1(ur[0], 0, 1, ks);
    };
    auto want_u1 = [&](int ks) __attribute__((always_inline)) { // ... and of the second
        if (NP != 1) {
            if (ks < 2) load_ub(ur[1], 1, ks);
            load_u1(ur[1], 1, 0, ks);
            load_u1(ur[1], 1, 1, ks);
        }
    };
    const std::true_type yes;
    const std::false_type no;
    // chunk 0 goes to LDS by itself
    write_x(x0, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) write_v(v0, 0, i);
    if (!MULTI && nch == 4) {
        // The common short contraction (512), spelled out: every chunk is requested exactly once, and the stage-2
        // operands follow in the last two chunks, when nothing else is left to ask for.
        load_x(x2, 2);
        load_x(x3, 3);
        load_v(v0, 2);
        __syncthreads();
        step(x1, v1, 0, no, [&](int ks) __attribute__((always_inline)) { load_v1(v1, 3, ks); });
        step(x2, v0, 1, no, none);
        step(x3, v1, 2, no, want_u0);
        step(x0, v0, 3, no, want_u1);
    } else {
        // Any length: requests are unconditional (a chunk past the end repeats the last one, and what it brings is
        // never multiplied), the stage-2 operands are asked for early.
        load_x(x2, 2);
        load_x(x3, 3);
        load_x(x0, 4);
        load_v(v0, 2);
        __syncthreads();
        step(x1, v1, 0, yes, want_u0);
        step(x2, v0, 1, yes, want_u1);
        step(x3, v1, 2, yes, none);
        step(x0, v0, 3, yes, none);
        for (int c = 4; c < nch; c += 4) {
            step(x1, v1, c, yes, none);
            step(x2, v0, c + 1, yes, none);
            step(x3, v1, c + 2, yes, none);
            step(x0, v0, c + 3, yes, none);
        }
    }

    // ---- intermediate -> LDS (bf16, row-major): lane holds row `col`, rho = 32 w + 8 q + 4 half + 0..3
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        u32x2_t pk;
        pk.x = pack_bf16x2(acc0[4 * q] + acc1[4 * q], acc0[4 * q + 1] + acc1[4 * q + 1]);
        pk.y = pack_bf16x2(acc0[4 * q + 2] + acc1[4 * q + 2], acc0[4 * q + 3] + acc1[4 * q + 3]);
        *(uint2_alias *)&Ts[col * LC_TP + 32 * w + 8 * q + 4 * half] = pk;
    }
    __syncthreads();
    if (a.mid_save) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = cr + 16 * i;
            if (row0 + r < a.rows)
                *(uint4_alias *)(a.mid_save + (row0 + r) * LC_R + 8 * co) = *(const uint4_alias *)&Ts[r * LC_TP + 8 * co];
        }
    }
    bf16x8_t tf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) tf[ks] = lc_as_bf16x8(*(const uint4_alias *)&Ts[col * LC_TP + 16 * ks + 8 * half]);

    // ---- stage 2: pairs of output blocks
    uint16_t *Us = &Vs[0][0] + w * (64 * LC_TP); // 64 rows of W2 per wavefront
    static_assert(4 * 64 * LC_TP <= 2 * LC_KC * LC_VP, "the W2 patches must fit in the W1 buffers");
    // rows of W2 -> MFMA fragments through this wavefront's patch of LDS (the W1 buffers are free by now): rows
    // 0..31 of the patch hold the first block of a pair, rows 32..63 the second.  While one half is multiplied the
    // other half is rewritten with the block that comes next (a wavefront's LDS accesses are performed in the order
    // it issues them, and the patch is its own: no barrier).
    auto write_u = [&](const UR &u, int bi, int j) __attribute__((always_inline)) {
        *(uint4_alias *)&Us[(32 * bi + 4 * j + (lane >> 4)) * LC_TP + 8 * (lane & 15)] = u.r[bi][j];
    };
    const u32x4_t one_k0 = {half == 0 ? 0x3f80u : 0u, 0u, 0u, 0u}; // the row [1 0 0 ...] that multiplies the bias
    auto mma_block = [&](const UR &u, int bi, f32x16_t &y, auto during) __attribute__((always_inline)) {
        u32x4_t uf[2];
        uf[0] = *(const uint4_alias *)&Us[(32 * bi + col) * LC_TP + 8 * half];
        y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lc_as_bf16x8(u32x4_t{u.b[bi], 0u, 0u, 0u}), lc_as_bf16x8(one_k0), y, 0, 0, 0);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks + 1 < 8) uf[(ks + 1) & 1] = *(const uint4_alias *)&Us[(32 * bi + col) * LC_TP + 16 * (ks + 1) + 8 * half];
            during(ks);
            y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lc_as_bf16x8(uf[ks & 1]), tf[ks], y, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // The finished sums of a pair do not leave at once: they are kept (yp) and turned into bf16, row-major through a
    // per-wavefront LDS patch, and stored, piece by piece between the MFMAs of the pair that follows (the conversion
    // is some 150 vector instructions of 4 cycles each, as long as the 16 MFMAs themselves), or in flush() at the end.
    f32x16_t yp[2];
    int obp = 0; // first output block of the pair held in yp
    u32x4_t ea[4], em[4], ov[4];
    // epilogue operands of the held pair: requested when the following pair starts, used 9 or more MFMAs later
    auto epi_operands = [&]() __attribute__((always_inline)) {
        if (EP && (a.ep_add || a.ep_mask)) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = lane + 64 * i, r = idx >> 3, ch = idx & 7;
                const i64 row = row0 + r < a.rows ? row0 + r : a.rows - 1;
                if (a.ep_add) ea[i] = *(const uint4_alias *)(a.ep_add + row * C2 + 32 * obp + 8 * ch);
                if (a.ep_mask) em[i] = *(const uint4_alias *)(a.ep_mask + row * C2 + 32 * obp + 8 * ch);
            }
        }
    };
    // piece s = 0..13 of the held pair's way out
    auto epi_slot = [&](int s) __attribute__((always_inline)) {
        if (s < 8) { // lane holds row `col`, outputs o = 32 (obp + bi) + 8 q + 4 half + 0..3
            const int bi = s >> 2, q = s & 3;
            u32x2_t pk;
            pk.x = pack_bf16x2(yp[bi][4 * q], yp[bi][4 * q + 1]);
            pk.y = pack_bf16x2(yp[bi][4 * q + 2], yp[bi][4 * q + 3]);
            *(uint2_alias *)&Ys[w][col * LC_YP + 32 * bi + 8 * q + 4 * half] = pk;
            return;
        }
        if (s == 8) __builtin_amdgcn_wave_barrier();
        // the patch [32 rows][64 outputs] leaves as 16-byte stores, 8 lanes per row: read in one slot, stored in the next
        if (s >= 9 && s <= 12) {
            const int i = s - 9, idx = lane + 64 * i, r = idx >> 3, ch = idx & 7;
            ov[i] = *(const uint4_alias *)&Ys[w][r * LC_YP + 8 * ch];
        }
        if (s >= 10 && s <= 13) {
            const int i = s - 10, idx = lane + 64 * i, r = idx >> 3, ch = idx & 7;
            u32x4_t v = ov[i];
            if (EP && (a.ep_add || a.ep_mask || a.ep_relu)) { // (uniform)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float lo = bf16_bits_to_float((uint16_t)v[e]), hi = bf16_bits_to_float((uint16_t)(v[e] >> 16));
                    if (a.ep_add) {
                        lo += bf16_bits_to_float((uint16_t)ea[i][e]);
                        hi += bf16_bits_to_float((uint16_t)(ea[i][e] >> 16));
                    }
                    if (a.ep_relu) {
                        lo = fmaxf(lo, 0.f);
                        hi = fmaxf(hi, 0.f);
                    }
                    if (a.ep_mask) {
                        lo = bf16_bits_to_float((uint16_t)em[i][e]) > 0.f ? lo : 0.f;
                        hi = bf16_bits_to_float((uint16_t)(em[i][e] >> 16)) > 0.f ? hi : 0.f;
                    }
                    v[e] = pack_bf16x2(lo, hi);
                }
            }
            if (row0 + r < a.rows) *(uint4_alias *)(a.out + (row0 + r) * C2 + 32 * obp + 8 * ch) = v;
        }
        if (s == 13) __builtin_amdgcn_wave_barrier();
    };
    auto flush = [&]() __attribute__((always_inline)) {
        epi_operands();
#pragma unroll
        for (int s = 0; s < 14; ++s) epi_slot(s);
    };
    // u: the pair in work (its first block is in the patch already); un: the pair after it; uf / gf: registers to
    // refill and the pair to request into them, one piece per MFMA (gf < 0: nothing); held: yp holds a pair
    auto pair = [&](const UR &u, const UR &un, UR &uf, int gf, int g, bool held) __attribute__((always_inline)) {
        const int ob0 = w * obw + 2 * pair_of(g);
        f32x16_t y[2];
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int v = 0; v < 16; ++v) y[bi][v] = summing ? ysum[g < NSUM ? g : 0][bi][v] : 0.f;
        if (held) epi_operands();
        mma_block(u, 0, y[0], [&](int ks) __attribute__((always_inline)) {
            write_u(u, 1, ks);
            if (gf >= 0 && ks == 0) load_ub(uf, gf, 0);
            if (gf >= 0) load_u1(uf, gf, 0, ks);
            if (held) epi_slot(ks);
        });
        // (past the last pair `un` holds a repeat of it: written, never read)
        mma_block(u, 1, y[1], [&](int ks) __attribute__((always_inline)) {
            write_u(un, 0, ks);
            if (gf >= 0 && ks == 0) load_ub(uf, gf, 1);
            if (gf >= 0) load_u1(uf, gf, 1, ks);
            if (held) epi_slot(8 + ks);
        });
        if (summing && gi + 1 < G) { // (uniform) not the last group: keep the sums, nothing leaves yet
#pragma unroll
            for (int bi = 0; bi < 2; ++bi) ysum[g < NSUM ? g : 0][bi] = y[bi];
            return;
        }
#pragma unroll
        for (int bi = 0; bi < 2; ++bi) yp[bi] = y[bi];
        obp = ob0;
        if (summing) flush(); // (the sums over the groups take the registers a held pair would need)
    };
#pragma unroll
    for (int j = 0; j < 8; ++j) write_u(ur[0], 0, j);
    if (NP > 0) {
#pragma unroll
        for (int g = 0; g < NP; ++g)
            pair(ur[g % 3], ur[(g + 1 < NP ? g + 1 : g) % 3], ur[(g + 2) % 3], g + 2 < NP ? g + 2 : -1, g,
                 g > 0 && !summing);
    } else { // any number of pairs: one pair ahead, requests past the end repeat the last pair
        for (int g = 0; 2 * g < obw; g += 2) {
            pair(ur[0], ur[1], ur[2], -1, g, g > 0);
            load_u(ur[0], g + 2);
            if (2 * (g + 1) < obw) pair(ur[1], ur[0], ur[2], -1, g + 1, true);
            load_u(ur[1], g + 3);
        }
    }
    if (!summing) flush();
    } // groups
}

bool linear_chain2_multi_supported(i64 n_in, i64 n_out, i64 r, int groups, bool sum_out)
{
    if (!linear_chain2_supported(n_in, n_out, r) || groups < 1 || groups > LC_MAX_GROUPS) return false;
    return !sum_out || n_out == 256 || n_out == 512;
}

bool linear_chain2_supported(i64 n_in, i64 n_out, i64 r)
{
    return r == LC_R && n_in > 0 && n_out > 0 && n_in % 256 == 0 && n_out % 256 == 0 && n_in <= (1 << 20) &&
           n_out <= (1 << 20);
}

int launch_linear_chain2(hipStream_t s, const char *name, const LinChainArgs &a)
{
    int st = PF_OK;
    if (a.rows <= 0) return st;
    if (!linear_chain2_supported(a.C1, a.C2, LC_R)) return PF_ERR_UNSUPPORTED;
    const i64 tiles = (a.rows + LC_ROWS - 1) / LC_ROWS;
    if (tiles > 0x7fffffffLL) return PF_ERR_SHAPE;
    const dim3 grid((unsigned)tiles), block(256);
    if (a.groups > 1) {
        if (!linear_chain2_multi_supported(a.C1, a.C2, LC_R, a.groups, a.sum_out != 0)) return PF_ERR_UNSUPPORTED;
        if (a.sum_out) {
            if (a.C2 == 256) {
                PF_LAUNCH(st, name, (linear_chain2_kernel<1, 2>), grid, block, s, a);
            } else {
                PF_LAUNCH(st, name, (linear_chain2_kernel<2, 2>), grid, block, s, a);
            }
            return st;
        }
        switch (a.C2 / 256) {
        case 1: PF_LAUNCH(st, name, (linear_chain2_kernel<1, 1>), grid, block, s, a); break;
        case 2: PF_LAUNCH(st, name, (linear_chain2_kernel<2, 1>), grid, block, s, a); break;
        case 4: PF_LAUNCH(st, name, (linear_chain2_kernel<4, 1>), grid, block, s, a); break;
        case 8: PF_LAUNCH(st, name, (linear_chain2_kernel<8, 1>), grid, block, s, a); break;
        default: PF_LAUNCH(st, name, (linear_chain2_kernel<0, 1>), grid, block, s, a); break;
        }
        return st;
    }
    if (a.ep_add || a.ep_mask || a.ep_relu) {
        switch (a.C2 / 256) {
        case 1: PF_LAUNCH(st, name, (linear_chain2_kernel<1, 0, true>), grid, block, s, a); break;
        case 2: PF_LAUNCH(st, name, (linear_chain2_kernel<2, 0, true>), grid, block, s, a); break;
        case 4: PF_LAUNCH(st, name, (linear_chain2_kernel<4, 0, true>), grid, block, s, a); break;
        case 8: PF_LAUNCH(st, name, (linear_chain2_kernel<8, 0, true>), grid, block, s, a); break;
        default: PF_LAUNCH(st, name, (linear_chain2_kernel<0, 0, true>), grid, block, s, a); break;
        }
        return st;
    }
    switch (a.C2 / 256) {
    case 1: PF_LAUNCH(st, name, linear_chain2_kernel<1>, grid, block, s, a); break;
    case 2: PF_LAUNCH(st, name, linear_chain2_kernel<2>, grid, block, s, a); break;
    case 4: PF_LAUNCH(st, name, linear_chain2_kernel<4>, grid, block, s, a); break;
    case 8: PF_LAUNCH(st, name, linear_chain2_kernel<8>, grid, block, s, a); break;
    default: PF_LAUNCH(st, name, linear_chain2_kernel<0>, grid, block, s, a); break;
    }
    return st;
}

} // namespace pf
