// A stack of factorized LSTM layers over a whole sequence (paper Section 2.3, eq. (2); the 2-layer language
// model of Appendix D), small batches, fp32.  Same arithmetic as running the layers one after the other, but
// scheduled as a wavefront: layer l at time t only needs layer l - 1 at time t and itself at time t - 1, so
// slot s = l + t of the forward pass handles every layer that has a step there in the SAME launches (backward:
// the mirror image).  A step of the recurrence is a chain of short, latency-bound launches; the wavefront makes
// that chain T + L - 1 slots long instead of T L.
//
// General schedule (any factor layout): per forward slot one launch for all T = (h Vh | x Vx) products, one for
// their slice sums, one for all z = T U^T products, one for the gates of all active layers; the input path of layer 0
// does not depend on any recurrence and is computed for all time steps up front; the input path of a higher layer
// reads the layer below at the same time step and rides in the slot's launches.  With one factor pair per path and
// r <= 512 the products that follow the slice sums and the gate arithmetic are one kernel in either direction
// (lstm_zgates_kernel, lstm_dhgates_kernel): three launches per slot.  All parameter gradients are formed once per
// layer over all T B rows after the backward wavefront.  The factors are copied once per call into the order the
// kernels read them in.  A single layer over a sequence (pf_lowrank_lstm_seq_*) is a stack of one layer.
#include <vector>

#include "pf_gemm.h"
#include "pf_skinny.h"
#include "pf_common.h"

namespace pf {

constexpr int ST_MAX_LAYERS = 4;
constexpr int ST_RANK_MMA_ROWS = 128; // T B from which the weight gradients go to the matrix unit

__device__ __forceinline__ float st_sigmoid(float z) { return 1.0f / (1.0f + expf(-z)); }

// ---- gates of all active layers of a slot (blockIdx.y = position in the list) ----
struct StackGatesFwd {
    const float *P[ST_MAX_LAYERS];     // pre-activation slices, [nslices][B x 4h]
    const float *bias[ST_MAX_LAYERS];  // nullable
    const float *zadd[ST_MAX_LAYERS];  // nullable: pre-activations computed up front (layer 0's input path)
    const float *c_prev[ST_MAX_LAYERS];
    float *h_out[ST_MAX_LAYERS], *c_out[ST_MAX_LAYERS], *gates[ST_MAX_LAYERS];
    int nslices[ST_MAX_LAYERS];
    int n, B, h;
};

__global__ __launch_bounds__(256) void lstm_stack_gates_fwd_kernel(StackGatesFwd a)
{
    const int q = blockIdx.y, h = a.h;
    const i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (i64)a.B * h) return;
    const int b = (int)(idx / h), j = (int)(idx % h);
    const i64 base = (i64)b * 4 * h + j, pcount = (i64)a.B * 4 * h;
    float z[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) z[g] = slices_at(a.P[q], a.nslices[q], pcount, base + (i64)g * h);
    if (a.bias[q]) {
#pragma unroll
        for (int g = 0; g < 4; ++g) z[g] += a.bias[q][j + (i64)g * h];
    }
    if (a.zadd[q]) {
#pragma unroll
        for (int g = 0; g < 4; ++g) z[g] += a.zadd[q][base + (i64)g * h];
    }
    const float ig = st_sigmoid(z[0]), fg = st_sigmoid(z[1]), gg = tanhf(z[2]), og = st_sigmoid(z[3]);
    const float c = fg * a.c_prev[q][idx] + ig * gg;
    float *gt = a.gates[q];
    gt[base] = ig;
    gt[base + h] = fg;
    gt[base + 2 * (i64)h] = gg;
    gt[base + 3 * (i64)h] = og;
    a.c_out[q][idx] = c;
    a.h_out[q][idx] = og * tanhf(c);
}

// dh_t of a layer = what arrives from above (a tensor, or slices of dTx V_x^T of the layer above) + what arrives
// from its own step t + 1 (a tensor for the last step, else slices of dTh V_h^T); then the gate derivatives.
struct StackGatesBwd {
    const float *gates[ST_MAX_LAYERS], *c_prev[ST_MAX_LAYERS], *c_out[ST_MAX_LAYERS];
    const float *dh_a[ST_MAX_LAYERS], *dh_b[ST_MAX_LAYERS];       // tensors [B x h], nullable
    const float *P1[ST_MAX_LAYERS], *P2[ST_MAX_LAYERS];           // slice sets [n][B x h], nullable when n == 0
    const float *dc_next[ST_MAX_LAYERS];                          // nullable
    float *dz[ST_MAX_LAYERS], *dc_prev[ST_MAX_LAYERS];
    int n1[ST_MAX_LAYERS], n2[ST_MAX_LAYERS];
    int n, B, h;
};

__global__ __launch_bounds__(256) void lstm_stack_gates_bwd_kernel(StackGatesBwd a)
{
    const int q = blockIdx.y, h = a.h;
    const i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (i64)a.B * h) return;
    const int b = (int)(idx / h), j = (int)(idx % h);
    const i64 base = (i64)b * 4 * h + j, pc = (i64)a.B * h;
    float dhv = (a.dh_a[q] ? a.dh_a[q][idx] : 0.f) + (a.dh_b[q] ? a.dh_b[q][idx] : 0.f);
    dhv += slices_at(a.P1[q], a.n1[q], pc, idx) + slices_at(a.P2[q], a.n2[q], pc, idx);
    const float *gt = a.gates[q];
    const float ig = gt[base], fg = gt[base + h], gg = gt[base + 2 * (i64)h], og = gt[base + 3 * (i64)h];
    const float tc = tanhf(a.c_out[q][idx]);
    const float dc = (a.dc_next[q] ? a.dc_next[q][idx] : 0.f) + dhv * og * (1.f - tc * tc);
    a.dc_prev[q][idx] = dc * fg;
    float *dz = a.dz[q];
    dz[base] = dc * gg * ig * (1.f - ig);
    dz[base + h] = dc * a.c_prev[q][idx] * fg * (1.f - fg);
    dz[base + 2 * (i64)h] = dc * ig * (1.f - gg * gg);
    dz[base + 3 * (i64)h] = dhv * tc * og * (1.f - og);
}

// ---- z = Th Uh^T (+ Tx Ux^T) and the gates in one kernel (one factor pair per path) ----
// A workgroup owns ZG_HU hidden units of one layer, i.e. 4 ZG_HU = 64 pre-activation columns, and the whole
// contraction, so no slice sums leave the chip and eq. (2) is applied where z is formed.  The rank-r activations of
// both paths are staged in LDS once (rows past B and columns past r as zeros: no masks in the loop); the factors
// come from a copy in the kernel's own order (lstm_zg_pack_kernel).  Column i of MFMA sub-tile e is gate
// 2 e + i / 16 of unit u0 + i % 16.  With both paths the wavefronts take (path, half of r), with one path a
// quarter of r each; their accumulators meet in LDS, in a fixed order.
constexpr int ZG_HU = 16;
constexpr int ZG_MAXR8 = 512;            // r rounded up to 8 may not exceed this
constexpr int ZG_MAXP = ZG_MAXR8 + 4;    // LDS row pitch in floats: r8 + 4
constexpr int ZG_CH = 4;                 // super-steps (of eight contraction indices) per prefetch stage
constexpr int ZG_NST = 4;                // prefetch stages

// Packed order of the fused kernels: for a workgroup's column tile and the eight contraction indices 8 S .. 8 S + 7,
// the 16 bytes of lane l for MFMA sub-tile e hold k = 8 S + 4 (l / 32) + 0..3 of one column, at float offset
// (((tile * ceil(r / 8) + S) * E + e) * 64 + l) * 4.  Source matrices are [columns][r] row-major.
//   mode 0 (E = 2, U[4h][r]): column l % 32 of sub-tile e is gate 2 e + (l % 32) / 16 of unit 16 tile + l % 16
//   mode 1 (E = 1, V[h][r]):  column l % 32 is unit 32 tile + l % 32
inline size_t zg_packed_floats(int h, int r, int mode)
{
    const int tiles = mode == 0 ? (h + ZG_HU - 1) / ZG_HU : (h + 31) / 32, E = mode == 0 ? 2 : 1;
    return (size_t)tiles * (size_t)((r + 7) / 8) * 256 * E;
}

struct ZgPackArgs {
    const float *src[2 * ST_MAX_LAYERS];
    float *dst[2 * ST_MAX_LAYERS];
    int n, h, r, mode;
};
// one thread per 16-byte item
__global__ __launch_bounds__(256) void lstm_zg_pack_kernel(ZgPackArgs a)
{
    const int S_total = (a.r + 7) / 8, E = a.mode == 0 ? 2 : 1;
    const int tiles = a.mode == 0 ? (a.h + ZG_HU - 1) / ZG_HU : (a.h + 31) / 32;
    const i64 per = (i64)tiles * S_total * 64 * E, g = (i64)blockIdx.x * 256 + threadIdx.x;
    if (g >= per * a.n) return;
    const int mi = (int)(g / per);
    const i64 it = g % per;
    const int lane = (int)(it & 63), e = (int)((it >> 6) % E);
    const int S = (int)((it / (64 * E)) % S_total), tile = (int)((it / (64 * E)) / S_total);
    const int i = lane & 31;
    const int unit = a.mode == 0 ? tile * ZG_HU + (i & 15) : tile * 32 + i;
    const i64 row = a.mode == 0 ? (i64)(2 * e + (i >> 4)) * a.h + unit : unit;
    f32x4_t v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const int k = 8 * S + 4 * (lane >> 5) + s4;
        if (k < a.r && unit < a.h) v[s4] = a.src[mi][row * a.r + k];
    }
    *(f32x4_t *)(a.dst[mi] + it * 4) = v;
}

// The products of a fused kernel: tot[e] += A_seg[32 x r] * W_seg(tile) over this wavefront's share of the
// contraction, for up to two (activations, factor) pairs.  NRI: rows a wavefront stages, ceil(B / 4) rounded up to
// 5 or 8; E: MFMA sub-tiles (32 columns each) of the workgroup's tile.  With two pairs the wavefronts take
// (pair, half of r), with one a quarter of r each, with none nothing.  Ends with the activations' LDS free again.
template <int NRI, int E>
__device__ __forceinline__ void fused_products(const float *A0, const float *A1, const float *W0, const float *W1,
                                               int nseg, int tile, int B, int r, float *lds, f32x16_t (&tot)[E])
{
    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, i = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6); // wavefront index, known to be uniform
    const int r8 = (r + 7) & ~7, P = r8 + 4, S_total = r8 / 8;

    // this wavefront's pair and range of super-steps
    int seg, S0, S1;
    if (nseg == 2) {
        const int per = (S_total + 1) / 2;
        seg = w >> 1;
        S0 = (w & 1) * per;
        S1 = min(S_total, S0 + per);
    } else {
        const int per = (S_total + 3) / 4;
        seg = 0;
        S0 = w * per;
        S1 = nseg == 0 ? S0 : min(S_total, S0 + per);
    }
    const float *Wp = (seg ? W1 : W0) + (i64)tile * S_total * (256 * E) + lane * 4; // + (S * E + e) * 256
    const float *Al = lds + (seg * 32 + i) * P + 4 * half;                          // + 8 S

    struct Stage {
        f32x4_t wv[ZG_CH][E];
    };
    auto load = [&](Stage &st, int c) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < ZG_CH; ++q) {
            const int S = min(S0 + c * ZG_CH + q, S_total - 1); // past the range: loaded, never used
#pragma unroll
            for (int e = 0; e < E; ++e) st.wv[q][e] = *(const f32x4_t *)(Wp + ((i64)S * E + e) * 256);
        }
    };
#pragma unroll
    for (int e = 0; e < E; ++e)
#pragma unroll
        for (int v = 0; v < 16; ++v) tot[e][v] = 0.f;
    // The activation fragments of a stage are read from LDS one stage ahead of their use; super-steps past the
    // wavefront's range read a valid address and multiply by zero.  A wavefront adds up at most 256 contraction
    // indices (half of r <= 512) in its accumulators, and the MFMAs follow each other without a pause: moving
    // accumulators out to add them elsewhere would leave the matrix unit idle for as long as eight MFMAs.
    auto lds_read = [&](f32x4_t(&av)[ZG_CH], int c) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < ZG_CH; ++q) {
            const int S = S0 + c * ZG_CH + q;
            const f32x4_t t = *(const f32x4_t *)(Al + 8 * min(S, S_total - 1));
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) av[q][s4] = S < S1 ? t[s4] : 0.f;
        }
    };
    auto compute = [&](const Stage &st, const f32x4_t(&av)[ZG_CH]) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < ZG_CH; ++q)
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                for (int e = 0; e < E; ++e)
                    tot[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][s4], st.wv[q][e][s4], tot[e], 0, 0, 0);
    };
    const int nch = S1 > S0 ? (S1 - S0 + ZG_CH - 1) / ZG_CH : 0;
    // activations -> LDS, 16 bytes per item (rows are only 4-byte aligned in memory): wavefront w takes rows
    // w, w + 4, ..., a lane the items lane and lane + 64 of a row (r8 <= 512 floats = 128 items).  Items inside a
    // row are loaded whole; the one item per row that straddles its end is filled float by float; rows past B and
    // columns past r are written as zeros.
    struct __attribute__((packed, aligned(4))) F4 {
        float f[4];
    };
    auto stage_load = [&](f32x4_t(&v)[2 * NRI], const float *A) __attribute__((always_inline)) {
#pragma unroll
        for (int ri = 0; ri < NRI; ++ri)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = w + 4 * ri, k4 = 4 * (lane + 64 * j);
                const bool inside = row < B && k4 + 3 < r;
                const F4 t = *(const F4 *)(A + (inside ? (i64)row * r + k4 : 0));
                v[2 * ri + j] = f32x4_t{t.f[0], t.f[1], t.f[2], t.f[3]};
            }
    };
    auto stage_store = [&](const f32x4_t(&v)[2 * NRI], int sg) __attribute__((always_inline)) {
#pragma unroll
        for (int ri = 0; ri < NRI; ++ri)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = w + 4 * ri, k4 = 4 * (lane + 64 * j);
                const bool inside = row < B && k4 + 3 < r, straddles = row < B && k4 < r && k4 + 3 >= r;
                f32x4_t o;
#pragma unroll
                for (int c = 0; c < 4; ++c) o[c] = inside ? v[2 * ri + j][c] : 0.f;
                if (k4 < r8 && !straddles) *(f32x4_t *)&lds[(sg * 32 + row) * P + k4] = o;
            }
    };
    // Every wavefront has the compute unit's SIMD to itself and only its loads hide the memory latency, so all of
    // them are requested before the first wait: a ring of ZG_NST stages of factors (16 super-steps; the first fill
    // is unconditional so that the loads in flight can be counted exactly), the activations (both pairs when a
    // wavefront stages at most five rows, i.e. B <= 20) and the item that straddles the end of a row.
    Stage st[ZG_NST];
    {
        constexpr bool BOTH = NRI <= 5;
        f32x4_t v[2 * NRI], v2[BOTH ? 2 * NRI : 1];
#pragma unroll
        for (int d = 0; d < ZG_NST; ++d) load(st[d], d);
        stage_load(v, A0);
        if constexpr (BOTH) stage_load(v2, A1); // (with fewer than two pairs A1 == A0: loaded, not stored)
        const int k4t = r & ~3; // the straddling item of a row, if r is not a multiple of four
        const bool fix = tid < nseg * 32 && (tid & 31) < B && k4t < r;
        const float *src = ((tid >> 5) && nseg == 2 ? A1 : A0) + (fix ? (i64)(tid & 31) * r + k4t : 0);
        f32x4_t o = {src[0], 0.f, 0.f, 0.f};
        const float o1 = src[fix && k4t + 1 < r ? 1 : 0], o2 = src[fix && k4t + 2 < r ? 2 : 0];
        stage_store(v, 0);
        if (nseg == 2) {
            if constexpr (!BOTH) {
                stage_load(v, A1);
                stage_store(v, 1);
            } else {
                stage_store(v2, 1);
            }
        }
        // rows this wavefront does not reach with NRI rows (none when NRI covers ceil(B / 4)) stay unwritten only
        // if they are past row 4 NRI + 3: write their zeros
        for (int row = 4 * NRI + w; row < 32; row += 4)
            for (int sg = 0; sg < nseg; ++sg)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int k4 = 4 * (lane + 64 * j);
                    if (k4 < r8) *(f32x4_t *)&lds[(sg * 32 + row) * P + k4] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                }
        if (fix) {
            o[1] = k4t + 1 < r ? o1 : 0.f;
            o[2] = k4t + 2 < r ? o2 : 0.f;
            *(f32x4_t *)&lds[((tid >> 5) * 32 + (tid & 31)) * P + k4t] = o;
        }
    }
    __syncthreads(); // the staged activations are complete
    static_assert(ZG_NST % 2 == 0, "the two fragment buffers alternate with the stage index");
    f32x4_t av[2][ZG_CH];
    lds_read(av[0], 0);
    for (int c = 0; c < nch; c += ZG_NST) {
#pragma unroll
        for (int d = 0; d < ZG_NST; ++d) {
            if (c + d < nch) { // uniform; the body is one straight run of instructions
                // next stage's fragments, this stage's MFMAs, and the refill of this stage's registers (past the
                // range: a repeat of the last valid address).  Program order would issue the reads and the
                // refill after the last MFMA and leave the matrix unit idle meanwhile: the groups below ask the
                // scheduler to deal them out between the MFMAs instead.
                lds_read(av[(d + 1) & 1], c + d + 1);
                Stage nx;
                load(nx, c + d + ZG_NST);
                compute(st[d], av[d & 1]);
                st[d] = nx;
#define ZG_DEAL(ds)                                       \
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);    \
    __builtin_amdgcn_sched_group_barrier(0x100, ds, 0);   \
    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);    \
    __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                ZG_DEAL(1) ZG_DEAL(1) ZG_DEAL(1) ZG_DEAL(1)
                if constexpr (E == 2) {
                    ZG_DEAL(0) ZG_DEAL(0) ZG_DEAL(0) ZG_DEAL(0)
                }
#undef ZG_DEAL
            }
        }
    }
}

// The four wavefronts' tiles meet in LDS as red[4][E][16][64] (accumulator element v of lane l is row
// 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32); the sum of a (row m, sub-tile e, column i) over the wavefronts, in
// a fixed order, is fused_sum.
template <int E>
__device__ __forceinline__ void fused_exchange(float *lds, const f32x16_t (&tot)[E])
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    __syncthreads(); // the activations are no longer needed
#pragma unroll
    for (int e = 0; e < E; ++e)
#pragma unroll
        for (int v = 0; v < 16; ++v) lds[((w * E + e) * 16 + v) * 64 + lane] = tot[e][v];
    __syncthreads();
}
template <int E>
__device__ __forceinline__ float fused_sum(const float *red, int m, int e, int i)
{
    const int at = (e * 16 + (((m >> 3) << 2) | (m & 3))) * 64 + ((m >> 2) & 1) * 32 + i;
    return (red[at] + red[E * 1024 + at]) + (red[2 * E * 1024 + at] + red[3 * E * 1024 + at]);
}

struct ZgLayer {
    const float *A[2];  // [B x r] activations of the hidden path and of the input path
    const float *W[2];  // their factors, packed (mode 0)
    const float *bias, *zadd, *c_prev; // bias, zadd nullable
    float *h_out, *c_out, *gates;
    int nseg, wg0;
};
struct ZgArgs {
    ZgLayer l[ST_MAX_LAYERS];
    int n, B, h, r, tiles;
};

template <int NRI>
__global__ __launch_bounds__(256, 1) void lstm_zgates_kernel(ZgArgs a)
{
    __shared__ __attribute__((aligned(16))) float lds[2 * 32 * ZG_MAXP];
    int li = 0;
#pragma unroll
    for (int x = 1; x < ST_MAX_LAYERS; ++x)
        if (x < a.n && (int)blockIdx.x >= a.l[x].wg0) li = x;
    const ZgLayer &L = a.l[li];
    const int tile = blockIdx.x - L.wg0, tid = threadIdx.x;
    const int B = a.B, h = a.h;
    // both paths' pointers are read once as scalars and chosen per lane (indexing the argument block with a
    // per-lane index would turn every use into a dependent memory read)
    const float *A0 = L.A[0], *A1 = L.nseg == 2 ? L.A[1] : L.A[0];
    const float *W0 = L.W[0], *W1 = L.nseg == 2 ? L.W[1] : L.W[0];
    f32x16_t tot[2];
    fused_products<NRI, 2>(A0, A1, W0, W1, L.nseg, tile, B, a.r, lds, tot);

    // the operands of the gate arithmetic are fetched while the tiles are exchanged (at most two elements per thread)
    float pre_c[2], pre_b[2][4], pre_z[2][4];
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int el = tid + 256 * it, m = el / ZG_HU, unit = tile * ZG_HU + el % ZG_HU;
        const bool ok = el < B * ZG_HU && unit < h;
        const i64 base = ok ? (i64)m * 4 * h + unit : 0, idx = ok ? (i64)m * h + unit : 0;
        pre_c[it] = L.c_prev[idx];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            pre_b[it][g] = L.bias ? L.bias[(i64)g * h + (ok ? unit : 0)] : 0.f;
            pre_z[it][g] = L.zadd ? L.zadd[base + (i64)g * h] : 0.f;
        }
    }
    fused_exchange<2>(lds, tot);
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int el = tid + 256 * it, m = el / ZG_HU, u = el % ZG_HU, unit = tile * ZG_HU + u;
        if (el >= B * ZG_HU || unit >= h) continue;
        const i64 base = (i64)m * 4 * h + unit, idx = (i64)m * h + unit;
        float z[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) z[g] = (fused_sum<2>(lds, m, g >> 1, (g & 1) * 16 + u) + pre_b[it][g]) + pre_z[it][g];
        const float ig = st_sigmoid(z[0]), fg = st_sigmoid(z[1]), gg = tanhf(z[2]), og = st_sigmoid(z[3]);
        const float c = fg * pre_c[it] + ig * gg;
        L.gates[base] = ig;
        L.gates[base + h] = fg;
        L.gates[base + 2 * (i64)h] = gg;
        L.gates[base + 3 * (i64)h] = og;
        L.c_out[idx] = c;
        L.h_out[idx] = og * tanhf(c);
    }
}

// ---- backward: dh_t = (what arrives from above and from the final state) + dTh_{t+1} Vh^T + dTx^{above}_t Vx^{above T},
// then the gate derivatives, in one kernel.  A workgroup owns 32 hidden units of a layer and the whole contraction of
// both products; the rank-r gradients are tensors by then (their slice sums were formed in the slot before).  With
// dh_out set the sum is written there instead (the gradient that reaches a layer's initial state).
struct DgLayer {
    const float *A[2];  // [B x r]: this layer's dTh at t + 1 and / or the dTx of the layer above at t (nseg of them)
    const float *W[2];  // packed (mode 1) Vh of this layer / Vx of the layer above
    const float *dh_a, *dh_b;                       // [B x h] addends, nullable
    const float *gates, *c_prev, *c_out, *dc_next;  // dc_next nullable
    float *dz, *dc_prev, *dh_out;
    int nseg, wg0;
};
struct DgArgs {
    DgLayer l[ST_MAX_LAYERS];
    int n, B, h, r, tiles;
};

template <int NRI>
__global__ __launch_bounds__(256, 1) void lstm_dhgates_kernel(DgArgs a)
{
    __shared__ __attribute__((aligned(16))) float lds[2 * 32 * ZG_MAXP];
    int li = 0;
#pragma unroll
    for (int x = 1; x < ST_MAX_LAYERS; ++x)
        if (x < a.n && (int)blockIdx.x >= a.l[x].wg0) li = x;
    const DgLayer &L = a.l[li];
    const int tile = blockIdx.x - L.wg0, tid = threadIdx.x;
    const int B = a.B, h = a.h;
    const float *A0 = L.A[0], *A1 = L.nseg == 2 ? L.A[1] : L.A[0];
    const float *W0 = L.W[0], *W1 = L.nseg == 2 ? L.W[1] : L.W[0];
    f32x16_t tot[1];
    fused_products<NRI, 1>(A0, A1, W0, W1, L.nseg, tile, B, a.r, lds, tot);

    // operands of the gate derivatives, fetched while the tiles are exchanged (B * 32 <= 1024 elements: four per thread)
    const bool gates_on = L.dh_out == nullptr;
    float pa[4], pg[4][4], pcp[4], pco[4], pdc[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int el = tid + 256 * it, m = el >> 5, unit = tile * 32 + (el & 31);
        const bool ok = el < B * 32 && unit < h;
        const i64 base = ok ? (i64)m * 4 * h + unit : 0, idx = ok ? (i64)m * h + unit : 0;
        pa[it] = (L.dh_a ? L.dh_a[idx] : 0.f) + (L.dh_b ? L.dh_b[idx] : 0.f);
        if (gates_on) {
#pragma unroll
            for (int g = 0; g < 4; ++g) pg[it][g] = L.gates[base + (i64)g * h];
            pcp[it] = L.c_prev[idx];
            pco[it] = L.c_out[idx];
            pdc[it] = L.dc_next ? L.dc_next[idx] : 0.f;
        }
    }
    fused_exchange<1>(lds, tot);
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int el = tid + 256 * it, m = el >> 5, u = el & 31, unit = tile * 32 + u;
        if (el >= B * 32 || unit >= h) continue;
        const i64 base = (i64)m * 4 * h + unit, idx = (i64)m * h + unit;
        const float dhv = pa[it] + fused_sum<1>(lds, m, 0, u);
        if (!gates_on) {
            L.dh_out[idx] = dhv;
            continue;
        }
        const float ig = pg[it][0], fg = pg[it][1], gg = pg[it][2], og = pg[it][3];
        const float tc = tanhf(pco[it]);
        const float dc = pdc[it] + dhv * og * (1.f - tc * tc);
        L.dc_prev[idx] = dc * fg;
        L.dz[base] = dc * gg * ig * (1.f - ig);
        L.dz[base + h] = dc * pcp[it] * fg * (1.f - fg);
        L.dz[base + 2 * (i64)h] = dc * ig * (1.f - gg * gg);
        L.dz[base + 3 * (i64)h] = dhv * tc * og * (1.f - og);
    }
}

static bool zg_supported(int G, int r) { return G == 1 && ((r + 7) & ~7) <= ZG_MAXR8; }

// ---- a launch (or a few) of skinny products whose slice sums are laid out region by region ----
// Problems of one region write different columns of the same slices (the four gate blocks of a z product), so
// they must get the same slicing: same K, same launch.
struct SkItem {
    SkinnyProb p;
    int region;
    i64 coloff;
};
struct SkBatch {
    std::vector<SkItem> items;
    std::vector<size_t> region_off, region_len; // floats, filled by run()
    std::vector<int> region_ksplit;
    int nregions = 0;
    int new_region() { return nregions++; }
    void add(const SkinnyProb &p, int region, i64 coloff = 0) { items.push_back(SkItem{p, region, coloff}); }
    // Plans every launch (at most SK_MAX_PROB problems each, regions kept whole), places the slices from `part`
    // on (NULL: sizes only; cap floats are there) and launches unless dry.  *used: the floats of `part` taken.
    int run(hipStream_t s, const char *name, bool nk, float *part, size_t cap, bool dry, size_t *used, bool packed = true)
    {
        region_off.assign(nregions, 0);
        region_len.assign(nregions, 0);
        region_ksplit.assign(nregions, 0);
        std::vector<SkinnyArgs> launches;
        size_t off = 0, i = 0;
        while (i < items.size()) {
            // the chunk: whole regions while they fit
            size_t j = i;
            while (j < items.size()) {
                size_t k = j;
                while (k < items.size() && items[k].region == items[j].region) ++k;
                if (k - i > (size_t)SK_MAX_PROB) break;
                j = k;
            }
            if (j == i) return PF_ERR_UNSUPPORTED; // a region larger than a launch
            SkinnyArgs a = {};
            for (size_t k = i; k < j; ++k) a.p[a.nprob++] = items[k].p;
            skinny_plan(a);
            for (size_t k = i; k < j; ++k) {
                const SkinnyProb &pl = a.p[k - i];
                const int r = items[k].region;
                const size_t len = (size_t)pl.ksplit * (size_t)pl.pcount;
                if (region_ksplit[r] == 0) {
                    region_ksplit[r] = pl.ksplit;
                    region_len[r] = len;
                    region_off[r] = off;
                    off += len;
                } else if (region_ksplit[r] != pl.ksplit || region_len[r] != len) {
                    return PF_ERR_UNSUPPORTED;
                }
                a.p[k - i].P = part ? part + region_off[r] + items[k].coloff : nullptr;
            }
            launches.push_back(a);
            i = j;
        }
        if (used) *used = off;
        if (dry) return PF_OK;
        if (!part || off > cap) return PF_ERR_WORKSPACE;
        int st = PF_OK;
        for (size_t q = 0; q < launches.size() && st == PF_OK; ++q)
            st = packed ? launch_skinny_gemm_packed(s, name, launches[q]) : launch_skinny_gemm(s, name, launches[q], nk);
        return st;
    }
};

struct StackGeom {
    int T, B, din, h, r, G, gr, L;
    bool has_bias;
};

static int check_stack_desc(const pf_lstm_stack_desc *d, StackGeom *g)
{
    if (!d) return PF_ERR_NULL;
    if (d->dtype != PF_F32) return PF_ERR_UNSUPPORTED;
    if (d->groups != 1 && d->groups != 4) return PF_ERR_UNSUPPORTED;
    if (d->T < 0 || d->B < 0 || d->d_in <= 0 || d->h <= 0 || d->r <= 0) return PF_ERR_SHAPE;
    if (d->layers < 1 || d->layers > ST_MAX_LAYERS) return PF_ERR_SHAPE;
    const i64 lim = 0x7fffffffLL;
    if (d->T > lim || d->B > lim || d->d_in > lim || d->h > lim / 4 || d->r > lim / 4) return PF_ERR_SHAPE;
    if (d->T * d->B > lim || d->T * d->B * d->h * 4 > (lim << 3) || d->T * d->B * d->d_in > (lim << 3)) return PF_ERR_SHAPE;
    // built on the few-row streaming products: B <= 32 and every extent at least 4
    if (d->T > 0 && d->B > 0 && (d->B > SK_MAX_ROWS || d->d_in < 4 || d->h < 4 || d->r < 4)) return PF_ERR_UNSUPPORTED;
    if (g)
        *g = StackGeom{(int)d->T, (int)d->B, (int)d->d_in, (int)d->h, (int)d->r, d->groups, (int)(d->groups * d->r),
                       d->layers, d->has_bias != 0};
    return PF_OK;
}

// C[Mt x N] = A[Mt x K] W (+ bias) for Mt = T B rows, 512 rows per launch pair (product + slice sums)
constexpr int ST_ROWS = SK_MAX_ROWS * SK_MAX_PROB;
static int st_tall(hipStream_t s, const char *name, bool nk, i64 Mt, const float *A, i64 lda, const float *W, i64 ldw,
                   int K, int N, float *out, i64 ldo, const float *bias, float *part)
{
    int st = PF_OK;
    for (i64 m0 = 0; m0 < Mt && st == PF_OK; m0 += ST_ROWS) {
        const int Mg = (int)(Mt - m0 < ST_ROWS ? Mt - m0 : ST_ROWS);
        SkinnyArgs a;
        skinny_rows(Mg, A + m0 * lda, lda, W, ldw, K, N, part, a);
        st = launch_skinny_gemm(s, name, a, nk);
        if (st != PF_OK) break;
        SliceSumArgs ss = {};
        ss.s[ss.nseg++] = skinny_rows_seg(a, Mg, out + m0 * ldo, ldo, bias);
        st = launch_slice_sum(s, ss);
    }
    return st;
}
static size_t st_tall_part(i64 Mt, int K, int N)
{
    SkinnyArgs a;
    size_t m = 0;
    const int full = (int)(Mt < ST_ROWS ? Mt : ST_ROWS), last = (int)(Mt % ST_ROWS);
    if (full > 0) m = skinny_rows(full, nullptr, K, nullptr, N, K, N, nullptr, a);
    if (last > 0) {
        const size_t v = skinny_rows(last, nullptr, K, nullptr, N, K, N, nullptr, a);
        if (v > m) m = v;
    }
    return m;
}

// slice sums of several regions, four segments per launch
static int st_slice_sums(hipStream_t s, const std::vector<SliceSumSeg> &segs, const char *name)
{
    int st = PF_OK;
    for (size_t i = 0; i < segs.size() && st == PF_OK; i += 4) {
        SliceSumArgs ss = {};
        for (size_t k = i; k < segs.size() && k < i + 4; ++k) ss.s[ss.nseg++] = segs[k];
        st = launch_slice_sum(s, ss, name);
    }
    return st;
}
static SliceSumSeg st_seg(const float *P, i64 pcount, int ldp, int ksplit, int M, int N, float *out, i64 ldo)
{
    SliceSumSeg sg;
    sg.P = P;
    sg.bias = nullptr;
    sg.out = out;
    sg.pcount = pcount;
    sg.ldo = ldo;
    sg.M = M;
    sg.ldp = ldp;
    sg.ksplit = ksplit;
    sg.N = N;
    return sg;
}

// Per-layer tensors of the two entry points (host arrays of device pointers, copied)
struct StackPtrs {
    const float *h0[ST_MAX_LAYERS], *c0[ST_MAX_LAYERS];
    const float *Vx[ST_MAX_LAYERS], *Ux[ST_MAX_LAYERS], *Vh[ST_MAX_LAYERS], *Uh[ST_MAX_LAYERS], *bias[ST_MAX_LAYERS];
    float *h_all[ST_MAX_LAYERS], *c_all[ST_MAX_LAYERS], *gates_all[ST_MAX_LAYERS], *Tx_all[ST_MAX_LAYERS],
        *Th_all[ST_MAX_LAYERS];
};

// The factors in the order the streaming kernel reads them (see skinny_packed_floats), copied once per call: every
// one of the T + L - 1 slots reuses them.  Forward roles: T = a V (contraction over V's rows), z = T U^T (over U's
// columns); backward roles: dT = dz U (over U's rows), dh = dT V^T (over V's columns).
struct StackPacked {
    const float *Vh[ST_MAX_LAYERS], *Vx[ST_MAX_LAYERS];       // Vx: layers above the first only
    const float *Uh[ST_MAX_LAYERS][4], *Ux[ST_MAX_LAYERS][4]; // per gate block when every gate has its own pair
    const float *zg[ST_MAX_LAYERS][2];                        // forward, fused z + gates: Uh and Ux in that kernel's order
    const float *dg[ST_MAX_LAYERS][2];                        // backward, fused dh + gates: Vh and Vx in that kernel's order
    bool fused_z;                                             // either direction: the fused kernel of that direction is used
};
// Places the copies from buf on (NULL: sizes only), launches the copy kernels unless dry; returns the floats taken.
static size_t stack_pack(const StackGeom &g, const StackPtrs &p, bool bwd, float *buf, StackPacked *out, bool dry,
                         hipStream_t s, int *status)
{
    const int h = g.h, r = g.r, gr = g.gr, nq = g.G == 1 ? 1 : 4;
    const bool fused = zg_supported(g.G, r); // forward: U in the fused kernel's order; backward: V
    if (out) out->fused_z = fused;
    size_t off = 0;
    int st = PF_OK;
    SkinnyPackArgs pa = {};
    auto flush = [&]() {
        if (!dry && st == PF_OK && pa.n > 0) st = launch_skinny_pack(s, pa);
        pa = SkinnyPackArgs{};
    };
    auto add = [&](const float *src, i64 sk, i64 sn, int K, int N) -> const float * {
        float *dst = buf ? buf + off : nullptr;
        off += skinny_packed_floats(K, N);
        if (!dry) {
            skinny_pack_add(pa, src, sk, sn, K, N, dst);
            if (pa.n == SK_MAX_PACK) flush();
        }
        return dst;
    };
    for (int l = 0; l < g.L; ++l) {
        for (int path = 0; path < 2; ++path) { // 0: hidden path, 1: input path (hoisted for the first layer)
            if (path == 1 && l == 0) continue;
            const float *V = dry ? nullptr : (path ? p.Vx[l] : p.Vh[l]), *U = dry ? nullptr : (path ? p.Ux[l] : p.Uh[l]);
            // V is [h x gr]: forward contracts over its rows, backward over its columns
            if (!(bwd && fused)) {
                const float *pv = bwd ? add(V, 1, gr, gr, h) : add(V, gr, 1, h, gr);
                if (out) (path ? out->Vx : out->Vh)[l] = pv;
            }
            for (int q = 0; q < nq && !(!bwd && fused); ++q) {
                // U (or its gate block q) is [rows x r] with rows = 4h or h
                const int rows = g.G == 1 ? 4 * h : h;
                const float *Uq = U ? U + (i64)q * h * r : nullptr;
                const float *pu = bwd ? add(Uq, r, 1, rows, r) : add(Uq, 1, r, r, rows);
                if (out) (path ? out->Ux : out->Uh)[l][q] = pu;
            }
        }
    }
    flush();
    if (fused) {
        ZgPackArgs za = {};
        za.h = h;
        za.r = r;
        za.mode = bwd ? 1 : 0;
        for (int l = 0; l < g.L; ++l)
            for (int path = 0; path < 2; ++path) {
                // forward: both paths of every layer (the first layer's input path too);
                // backward: Vh of every layer, Vx of the layers above the first
                if (bwd && path == 1 && l == 0) continue;
                float *dst = buf ? buf + off : nullptr;
                off += zg_packed_floats(h, r, za.mode);
                if (out) (bwd ? out->dg : out->zg)[l][path] = dst;
                if (!dry) {
                    za.src[za.n] = bwd ? (path ? p.Vx[l] : p.Vh[l]) : (path ? p.Ux[l] : p.Uh[l]);
                    za.dst[za.n++] = dst;
                }
            }
        if (!dry && st == PF_OK && za.n > 0) {
            const i64 items = (i64)(zg_packed_floats(h, r, za.mode) / 4) * za.n;
            PF_LAUNCH(st, "lstm_zg_pack", lstm_zg_pack_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), s, za);
        }
    }
    if (status) *status = st;
    return off;
}

// ---- forward slot: products and gates of the layers in `mask` (layer l at time t = slot - l) ----
// part (NULL: sizes only) holds the slices of one launch group at a time.
static int stack_fwd_slot(const StackGeom &g, const StackPtrs &p, const StackPacked &pk, const float *zx0, int slot,
                          float *part, size_t cap,
                          bool dry, hipStream_t s, size_t *need)
{
    const int B = g.B, h = g.h, r = g.r, G = g.G, gr = g.gr;
    const i64 Bh = (i64)B * h;
    int st = PF_OK;
    size_t used = 0, most = 0;
    // T = h_{t-1} Vh, and for layers above the first T = x_t Vx with x_t = the layer below at time t
    SkBatch kn;
    int reg_th[ST_MAX_LAYERS], reg_tx[ST_MAX_LAYERS];
    for (int l = 0; l < g.L; ++l) {
        const int t = slot - l;
        reg_th[l] = reg_tx[l] = -1;
        if (t < 0 || t >= g.T) continue;
        const float *hp = dry ? nullptr : (t ? p.h_all[l] + (i64)(t - 1) * Bh : p.h0[l]);
        reg_th[l] = kn.new_region();
        kn.add(skinny_prob(B, hp, h, pk.Vh[l], gr, h, gr, gr, (i64)B * gr), reg_th[l]);
        if (l > 0) {
            reg_tx[l] = kn.new_region();
            kn.add(skinny_prob(B, dry ? nullptr : p.h_all[l - 1] + (i64)t * Bh, h, pk.Vx[l], gr, h, gr, gr, (i64)B * gr),
                   reg_tx[l]);
        }
    }
    st = kn.run(s, "lstm_stack_T", false, part, cap, dry, &used);
    if (st != PF_OK) return st;
    most = used;
    if (!dry) {
        std::vector<SliceSumSeg> segs;
        for (int l = 0; l < g.L; ++l) {
            const int t = slot - l;
            if (reg_th[l] >= 0)
                segs.push_back(st_seg(part + kn.region_off[reg_th[l]], (i64)B * gr, gr, kn.region_ksplit[reg_th[l]], B, gr,
                                      p.Th_all[l] + (i64)t * B * gr, gr));
            if (reg_tx[l] >= 0)
                segs.push_back(st_seg(part + kn.region_off[reg_tx[l]], (i64)B * gr, gr, kn.region_ksplit[reg_tx[l]], B, gr,
                                      p.Tx_all[l] + (i64)t * B * gr, gr));
        }
        st = st_slice_sums(s, segs, "lstm_stack_T_sum");
        if (st != PF_OK) return st;
    }
    if (pk.fused_z) { // z and the gates in one launch, one workgroup per ZG_HU hidden units of a layer
        if (need) *need = most;
        if (dry) return st;
        ZgArgs za = {};
        za.B = B;
        za.h = h;
        za.r = r;
        za.tiles = (h + ZG_HU - 1) / ZG_HU;
        int wg = 0;
        for (int l = 0; l < g.L; ++l) {
            const int t = slot - l;
            if (t < 0 || t >= g.T) continue;
            ZgLayer &zl = za.l[za.n++];
            // Both paths for every layer: the first layer's Tx is known for all steps beforehand, but forming its
            // share of z here costs nothing extra (its workgroups would otherwise finish before the others) and
            // spares the product over all T B rows.
            zl.nseg = 2;
            zl.A[0] = p.Th_all[l] + (i64)t * B * gr;
            zl.W[0] = pk.zg[l][0];
            zl.A[1] = p.Tx_all[l] + (i64)t * B * gr;
            zl.W[1] = pk.zg[l][1];
            zl.bias = g.has_bias ? p.bias[l] : nullptr;
            zl.zadd = nullptr;
            zl.c_prev = t ? p.c_all[l] + (i64)(t - 1) * Bh : p.c0[l];
            zl.h_out = p.h_all[l] + (i64)t * Bh;
            zl.c_out = p.c_all[l] + (i64)t * Bh;
            zl.gates = p.gates_all[l] + (i64)t * B * 4 * h;
            zl.wg0 = wg;
            wg += za.tiles;
        }
        if (B <= 20) {
            PF_LAUNCH(st, "lstm_stack_z_gates", lstm_zgates_kernel<5>, dim3((unsigned)wg), dim3(256), s, za);
        } else {
            PF_LAUNCH(st, "lstm_stack_z_gates", lstm_zgates_kernel<8>, dim3((unsigned)wg), dim3(256), s, za);
        }
        return st;
    }
    // z slices = Th Uh^T (and Tx Ux^T above the first layer), one region per product, a layer's regions adjacent
    SkBatch nk;
    int reg_zh[ST_MAX_LAYERS], reg_zx[ST_MAX_LAYERS];
    const i64 pcz = (i64)B * 4 * h;
    auto add_z = [&](int region, const float *Tm, const float *const *U) { // U: the packed gate blocks
        if (G == 1) {
            nk.add(skinny_prob(B, Tm, gr, U[0], r, r, 4 * h, 4 * h, pcz), region);
        } else {
            for (int q = 0; q < 4; ++q)
                nk.add(skinny_prob(B, Tm ? Tm + (i64)q * r : nullptr, gr, U[q], r, r, h, 4 * h, pcz), region, (i64)q * h);
        }
    };
    for (int l = 0; l < g.L; ++l) {
        const int t = slot - l;
        reg_zh[l] = reg_zx[l] = -1;
        if (t < 0 || t >= g.T) continue;
        reg_zh[l] = nk.new_region();
        add_z(reg_zh[l], dry ? nullptr : p.Th_all[l] + (i64)t * B * gr, pk.Uh[l]);
        if (l > 0) {
            reg_zx[l] = nk.new_region();
            add_z(reg_zx[l], dry ? nullptr : p.Tx_all[l] + (i64)t * B * gr, pk.Ux[l]);
        }
    }
    st = nk.run(s, "lstm_stack_z", true, part, cap, dry, &used);
    if (st != PF_OK) return st;
    if (used > most) most = used;
    if (need) *need = most;
    if (dry) return st;
    StackGatesFwd ga = {};
    ga.B = B;
    ga.h = h;
    for (int l = 0; l < g.L; ++l) {
        const int t = slot - l;
        if (t < 0 || t >= g.T) continue;
        const int q = ga.n++;
        ga.P[q] = part + nk.region_off[reg_zh[l]];
        ga.nslices[q] = nk.region_ksplit[reg_zh[l]] + (l > 0 ? nk.region_ksplit[reg_zx[l]] : 0);
        // (a layer's two regions were created one after the other, so their slices are adjacent)
        ga.bias[q] = (l > 0 && g.has_bias) ? p.bias[l] : nullptr; // layer 0's bias is inside zx0
        ga.zadd[q] = l == 0 ? zx0 + (i64)t * pcz : nullptr;
        ga.c_prev[q] = t ? p.c_all[l] + (i64)(t - 1) * Bh : p.c0[l];
        ga.h_out[q] = p.h_all[l] + (i64)t * Bh;
        ga.c_out[q] = p.c_all[l] + (i64)t * Bh;
        ga.gates[q] = p.gates_all[l] + (i64)t * pcz;
    }
    const dim3 grid((unsigned)((Bh + 255) / 256), (unsigned)ga.n);
    PF_LAUNCH(st, "lstm_stack_gates_fwd", lstm_stack_gates_fwd_kernel, grid, dim3(256), s, ga);
    return st;
}

struct StackPlan {
    size_t n_zx0, n_part, n_part2, n_dT, n_dz, n_pack_f, n_pack_b, fwd_bytes, bwd_bytes;
};

// per-layer tensors of the backward pass
struct StackBwdPtrs {
    const float *dhT[ST_MAX_LAYERS], *dcT[ST_MAX_LAYERS];
    float *dh0[ST_MAX_LAYERS], *dc0[ST_MAX_LAYERS];
    float *dVx[ST_MAX_LAYERS], *dUx[ST_MAX_LAYERS], *dVh[ST_MAX_LAYERS], *dUh[ST_MAX_LAYERS], *dbias[ST_MAX_LAYERS];
    float *dz_all[ST_MAX_LAYERS], *dTh_all[ST_MAX_LAYERS], *dTx_all[ST_MAX_LAYERS]; // workspace
};

// ---- backward slot u: layer l at time t with (L - 1 - l) + (T - 1 - t) = u ----
// part: slices of the dT products (consumed by the slice sums of the same slot); part2: slices of dh_{t-1} and of
// the dx handed to the layer below, consumed by the gate kernel of the NEXT slot, whose layout `prev` records.
struct StackCarry {
    const float *P1[ST_MAX_LAYERS], *P2[ST_MAX_LAYERS]; // for layer l: recurrent slices / slices from layer l + 1
    int n1[ST_MAX_LAYERS], n2[ST_MAX_LAYERS];
};
static int stack_bwd_slot(const StackGeom &g, const StackPtrs &p, const StackPacked &pk, const StackBwdPtrs &b,
                          const float *dh_top, int u,
                          float *part, size_t cap, float *part2, size_t cap2, StackCarry &carry, bool dry, hipStream_t s,
                          size_t *need, size_t *need2)
{
    const int B = g.B, h = g.h, r = g.r, G = g.G, gr = g.gr, L = g.L, T = g.T;
    const i64 Bh = (i64)B * h, pcz = (i64)B * 4 * h;
    int st = PF_OK;
    auto time_of = [&](int l) { return T - 1 - (u - (L - 1 - l)); };
    auto active = [&](int l) {
        const int t = time_of(l);
        return t >= 0 && t < T;
    };
    const i64 pcT = (i64)B * gr;
    if (pk.fused_z && !dry) {
        // dh (both products, whole contraction) and the gate derivatives in one launch, one workgroup per 32 hidden
        // units of a layer; a layer whose step 0 was the slot before gets its dh_{-1} = dTh_0 Vh^T here
        DgArgs da = {};
        da.B = B;
        da.h = h;
        da.r = r;
        da.tiles = (h + 31) / 32;
        int wg = 0;
        for (int l = 0; l < L; ++l) {
            const int t = time_of(l);
            if (t < -1 || t >= T) continue;
            DgLayer &dl = da.l[da.n++];
            if (t + 1 < T) { // this layer's own step t + 1
                dl.A[dl.nseg] = b.dTh_all[l] + (i64)(t + 1) * pcT;
                dl.W[dl.nseg++] = pk.dg[l][0];
            }
            if (t >= 0 && l + 1 < L) { // the layer above at the same step
                dl.A[dl.nseg] = b.dTx_all[l + 1] + (i64)t * pcT;
                dl.W[dl.nseg++] = pk.dg[l + 1][1];
            }
            if (dl.nseg == 0) { // nothing to multiply: valid operands of the right size, never used
                dl.A[0] = p.Th_all[l] + (i64)t * pcT;
                dl.W[0] = pk.dg[l][0];
            }
            if (t < 0) {
                dl.dh_out = b.dh0[l];
            } else {
                dl.dh_a = l == L - 1 ? dh_top + (i64)t * Bh : nullptr; // the top layer's dL/dh_t comes from outside
                dl.dh_b = t == T - 1 ? b.dhT[l] : nullptr;
                dl.gates = p.gates_all[l] + (i64)t * pcz;
                dl.c_prev = t ? p.c_all[l] + (i64)(t - 1) * Bh : p.c0[l];
                dl.c_out = p.c_all[l] + (i64)t * Bh;
                // dc_t lives in dc0 between the steps of a layer (each element is read, then rewritten, by its own thread)
                dl.dc_next = t == T - 1 ? b.dcT[l] : b.dc0[l];
                dl.dz = b.dz_all[l] + (i64)t * pcz;
                dl.dc_prev = b.dc0[l];
            }
            dl.wg0 = wg;
            wg += da.tiles;
        }
        if (da.n > 0) {
            if (B <= 20) {
                PF_LAUNCH(st, "lstm_stack_dh_gates", lstm_dhgates_kernel<5>, dim3((unsigned)wg), dim3(256), s, da);
            } else {
                PF_LAUNCH(st, "lstm_stack_dh_gates", lstm_dhgates_kernel<8>, dim3((unsigned)wg), dim3(256), s, da);
            }
            if (st != PF_OK) return st;
        }
    }
    if (!pk.fused_z && !dry) {
        StackGatesBwd ga = {};
        ga.B = B;
        ga.h = h;
        for (int l = 0; l < L; ++l) {
            if (!active(l)) continue;
            const int t = time_of(l), q = ga.n++;
            ga.gates[q] = p.gates_all[l] + (i64)t * pcz;
            ga.c_prev[q] = t ? p.c_all[l] + (i64)(t - 1) * Bh : p.c0[l];
            ga.c_out[q] = p.c_all[l] + (i64)t * Bh;
            ga.dh_a[q] = l == L - 1 ? dh_top + (i64)t * Bh : nullptr; // the top layer's dL/dh_t comes from outside
            ga.dh_b[q] = t == T - 1 ? b.dhT[l] : nullptr;
            ga.P1[q] = carry.P1[l];
            ga.n1[q] = t == T - 1 ? 0 : carry.n1[l];
            ga.P2[q] = carry.P2[l];
            ga.n2[q] = l == L - 1 ? 0 : carry.n2[l];
            // dc_t lives in dc0 between the steps of a layer (each element is read, then rewritten, by its own thread)
            ga.dc_next[q] = t == T - 1 ? b.dcT[l] : b.dc0[l];
            ga.dz[q] = b.dz_all[l] + (i64)t * pcz;
            ga.dc_prev[q] = b.dc0[l];
        }
        const dim3 grid((unsigned)((Bh + 255) / 256), (unsigned)ga.n);
        PF_LAUNCH(st, "lstm_stack_gates_bwd", lstm_stack_gates_bwd_kernel, grid, dim3(256), s, ga);
        if (st != PF_OK) return st;
    }
    // dTh = dz Uh, and above the first layer dTx = dz Ux (layer 0's input path is done for all steps at the end)
    SkBatch kn;
    int reg_h[ST_MAX_LAYERS], reg_x[ST_MAX_LAYERS];
    auto add_dT = [&](int region, const float *dz, const float *const *U) { // U: the packed gate blocks
        if (G == 1) {
            kn.add(skinny_prob(B, dz, 4 * (i64)h, U[0], r, 4 * h, r, gr, pcT), region);
        } else {
            for (int q = 0; q < 4; ++q)
                kn.add(skinny_prob(B, dz ? dz + (i64)q * h : nullptr, 4 * (i64)h, U[q], r, h, r, gr, pcT), region,
                       (i64)q * r);
        }
    };
    for (int l = 0; l < L; ++l) {
        reg_h[l] = reg_x[l] = -1;
        if (!active(l)) continue;
        const int t = time_of(l);
        const float *dz = dry ? nullptr : b.dz_all[l] + (i64)t * pcz;
        reg_h[l] = kn.new_region();
        add_dT(reg_h[l], dz, pk.Uh[l]);
        if (l > 0) {
            reg_x[l] = kn.new_region();
            add_dT(reg_x[l], dz, pk.Ux[l]);
        }
    }
    size_t used = 0;
    st = kn.run(s, "lstm_stack_dT", false, part, cap, dry, &used);
    if (st != PF_OK) return st;
    if (need) *need = used;
    if (!dry) {
        std::vector<SliceSumSeg> segs;
        for (int l = 0; l < L; ++l) {
            if (!active(l)) continue;
            const int t = time_of(l);
            segs.push_back(st_seg(part + kn.region_off[reg_h[l]], pcT, gr, kn.region_ksplit[reg_h[l]], B, gr,
                                  b.dTh_all[l] + (i64)t * pcT, gr));
            if (l > 0)
                segs.push_back(st_seg(part + kn.region_off[reg_x[l]], pcT, gr, kn.region_ksplit[reg_x[l]], B, gr,
                                      b.dTx_all[l] + (i64)t * pcT, gr));
        }
        st = st_slice_sums(s, segs, "lstm_stack_dT_sum");
        if (st != PF_OK) return st;
    }
    if (pk.fused_z) { // the dh products are part of the next slot's fused launch
        if (need2) *need2 = 0;
        return st;
    }
    // slices of dh_{t-1} = dTh Vh^T for the layer itself and of dx_t = dTx Vx^T for the layer below
    SkBatch nk;
    int reg_dh[ST_MAX_LAYERS], reg_dx[ST_MAX_LAYERS];
    for (int l = 0; l < L; ++l) {
        reg_dh[l] = reg_dx[l] = -1;
        if (!active(l)) continue;
        const int t = time_of(l);
        reg_dh[l] = nk.new_region();
        nk.add(skinny_prob(B, dry ? nullptr : b.dTh_all[l] + (i64)t * pcT, gr, pk.Vh[l], gr, gr, h, h, Bh),
               reg_dh[l]);
        if (l > 0) {
            reg_dx[l] = nk.new_region();
            nk.add(skinny_prob(B, dry ? nullptr : b.dTx_all[l] + (i64)t * pcT, gr, pk.Vx[l], gr, gr, h, h, Bh),
                   reg_dx[l]);
        }
    }
    st = nk.run(s, "lstm_stack_dh", true, part2, cap2, dry, &used);
    if (st != PF_OK) return st;
    if (need2) *need2 = used;
    if (dry) return st;
    std::vector<SliceSumSeg> last;
    for (int l = 0; l < L; ++l) {
        if (!active(l)) continue;
        carry.P1[l] = part2 + nk.region_off[reg_dh[l]];
        carry.n1[l] = nk.region_ksplit[reg_dh[l]];
        if (l > 0) {
            carry.P2[l - 1] = part2 + nk.region_off[reg_dx[l]];
            carry.n2[l - 1] = nk.region_ksplit[reg_dx[l]];
        }
        if (time_of(l) == 0) // the gradient that reaches the layer's initial state
            last.push_back(st_seg(carry.P1[l], Bh, h, carry.n1[l], B, h, b.dh0[l], h));
    }
    return st_slice_sums(s, last, "lstm_stack_dh0_sum");
}

static int plan_stack(const StackGeom &g, StackPlan *out)
{
    StackPlan p = {};
    const i64 Mt = (i64)g.T * g.B;
    if (Mt == 0) {
        *out = p;
        return PF_OK;
    }
    p.n_dz = (size_t)(Mt * 4 * g.h);
    // pre-activations of the first layer's input path for all steps: the fused schedule forms them step by step
    p.n_zx0 = zg_supported(g.G, g.r) ? 0 : p.n_dz;
    p.n_dT = (size_t)(Mt * g.gr);
    size_t m = 0, m2 = 0;
    auto upd = [&](size_t v) {
        if (v > m) m = v;
    };
    upd(st_tall_part(Mt, g.din, g.gr));                    // Tx = X Vx, layer 0
    upd(st_tall_part(Mt, g.r, g.G == 1 ? 4 * g.h : g.h));  // zx = Tx Ux^T
    upd(st_tall_part(Mt, g.G == 1 ? 4 * g.h : g.h, g.r));  // dTx = dz Ux
    upd(st_tall_part(Mt, g.gr, g.din));                    // dx = dTx Vx^T
    StackPtrs none = {};
    StackPacked nonep = {};
    nonep.fused_z = zg_supported(g.G, g.r);
    StackBwdPtrs noneb = {};
    StackCarry carry = {};
    for (int slot = 0; slot < g.T + g.L - 1; ++slot) {
        // the sets of active layers repeat: every slot in the middle has all of them
        if (slot >= g.L && slot < g.T - 1) continue;
        size_t need = 0, need2 = 0;
        int st = stack_fwd_slot(g, none, nonep, nullptr, slot, nullptr, 0, true, nullptr, &need);
        if (st != PF_OK) return st;
        upd(need);
        st = stack_bwd_slot(g, none, nonep, noneb, nullptr, slot, nullptr, 0, nullptr, 0, carry, true, nullptr, &need, &need2);
        if (st != PF_OK) return st;
        upd(need);
        if (need2 > m2) m2 = need2;
    }
    p.n_part = m;
    p.n_part2 = m2;
    p.n_pack_f = stack_pack(g, none, false, nullptr, nullptr, true, nullptr, nullptr);
    p.n_pack_b = stack_pack(g, none, true, nullptr, nullptr, true, nullptr, nullptr);
    p.fwd_bytes = align_up(p.n_zx0 * sizeof(float)) + align_up(p.n_part * sizeof(float)) + align_up(p.n_pack_f * sizeof(float));
    p.bwd_bytes = (size_t)g.L * (align_up(p.n_dz * sizeof(float)) + 2 * align_up(p.n_dT * sizeof(float))) +
                  align_up(p.n_part * sizeof(float)) + align_up(p.n_part2 * sizeof(float)) +
                  align_up(p.n_pack_b * sizeof(float));
    *out = p;
    return PF_OK;
}

} // namespace pf

using namespace pf;

extern "C" {

size_t pf_lowrank_lstm_stack_fwd_workspace_bytes(const pf_lstm_stack_desc *d)
{
    StackGeom g;
    StackPlan p;
    if (check_stack_desc(d, &g) != PF_OK || plan_stack(g, &p) != PF_OK) return 0;
    return p.fwd_bytes;
}

size_t pf_lowrank_lstm_stack_bwd_workspace_bytes(const pf_lstm_stack_desc *d)
{
    StackGeom g;
    StackPlan p;
    if (check_stack_desc(d, &g) != PF_OK || plan_stack(g, &p) != PF_OK) return 0;
    return p.bwd_bytes;
}

int pf_lowrank_lstm_stack_fwd(const pf_lstm_stack_desc *d, const void *x, const void *const *h0, const void *const *c0,
                              const void *const *Vx, const void *const *Ux, const void *const *Vh,
                              const void *const *Uh, const void *const *bias, void *const *h_all, void *const *c_all,
                              void *const *gates_all, void *const *Tx_all, void *const *Th_all, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    StackGeom g;
    int st = check_stack_desc(d, &g);
    if (st != PF_OK) return st;
    if (!h0 || !c0 || !Vx || !Ux || !Vh || !Uh || (g.has_bias && !bias) || !h_all || !c_all || !gates_all || !Tx_all ||
        !Th_all)
        return PF_ERR_NULL;
    StackPtrs p = {};
    for (int l = 0; l < g.L; ++l) {
        if (!Vx[l] || !Ux[l] || !Vh[l] || !Uh[l] || (g.has_bias && !bias[l])) return PF_ERR_NULL;
        if (g.T > 0 && g.B > 0 && (!h0[l] || !c0[l] || !h_all[l] || !c_all[l] || !gates_all[l] || !Tx_all[l] || !Th_all[l]))
            return PF_ERR_NULL;
        if (any_misaligned({h0[l], c0[l], Vx[l], Ux[l], Vh[l], Uh[l], g.has_bias ? bias[l] : nullptr, h_all[l], c_all[l],
                            gates_all[l], Tx_all[l], Th_all[l]},
                           16))
            return PF_ERR_UNSUPPORTED;
        p.h0[l] = (const float *)h0[l];
        p.c0[l] = (const float *)c0[l];
        p.Vx[l] = (const float *)Vx[l];
        p.Ux[l] = (const float *)Ux[l];
        p.Vh[l] = (const float *)Vh[l];
        p.Uh[l] = (const float *)Uh[l];
        p.bias[l] = g.has_bias ? (const float *)bias[l] : nullptr;
        p.h_all[l] = (float *)h_all[l];
        p.c_all[l] = (float *)c_all[l];
        p.gates_all[l] = (float *)gates_all[l];
        p.Tx_all[l] = (float *)Tx_all[l];
        p.Th_all[l] = (float *)Th_all[l];
    }
    if (g.T == 0 || g.B == 0) return PF_OK;
    if (!x || any_misaligned({x}, 16)) return x ? PF_ERR_UNSUPPORTED : PF_ERR_NULL;
    StackPlan pl;
    st = plan_stack(g, &pl);
    if (st != PF_OK) return st;
    if (!workspace || workspace_bytes < pl.fwd_bytes) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    float *zx0 = ws.take<float>(pl.n_zx0);
    float *part = ws.take<float>(pl.n_part);
    float *packed = ws.take<float>(pl.n_pack_f);
    if (!ws.ok()) return PF_ERR_WORKSPACE;
    StackPacked pk = {};
    stack_pack(g, p, false, packed, &pk, false, s, &st);
    if (st != PF_OK) return st;
    const i64 Mt = (i64)g.T * g.B;
    const int h = g.h, r = g.r, gr = g.gr;
    // the input path of the first layer for every time step at once
    st = st_tall(s, "lstm_stack_Tx0=X*Vx", false, Mt, (const float *)x, g.din, p.Vx[0], gr, g.din, gr, p.Tx_all[0], gr,
                 nullptr, part);
    if (st != PF_OK) return st;
    if (pk.fused_z) {
        // z of the first layer's input path is formed inside the fused kernel, step by step
    } else if (g.G == 1) {
        st = st_tall(s, "lstm_stack_zx0=Tx*Uxt", true, Mt, p.Tx_all[0], gr, p.Ux[0], r, r, 4 * h, zx0, 4 * (i64)h,
                     p.bias[0], part);
    } else {
        for (int q = 0; q < 4 && st == PF_OK; ++q)
            st = st_tall(s, "lstm_stack_zx0=Tx*Uxt", true, Mt, p.Tx_all[0] + (i64)q * r, gr, p.Ux[0] + (i64)q * h * r, r, r,
                         h, zx0 + (i64)q * h, 4 * (i64)h, p.bias[0] ? p.bias[0] + (i64)q * h : nullptr, part);
    }
    for (int slot = 0; slot < g.T + g.L - 1 && st == PF_OK; ++slot)
        st = stack_fwd_slot(g, p, pk, zx0, slot, part, pl.n_part, false, s, nullptr);
    return st;
}

int pf_lowrank_lstm_stack_bwd(const pf_lstm_stack_desc *d, const void *x, const void *const *h0, const void *const *c0,
                              const void *const *h_all, const void *const *c_all, const void *const *gates_all,
                              const void *const *Tx_all, const void *const *Th_all, const void *const *Vx,
                              const void *const *Ux, const void *const *Vh, const void *const *Uh, const void *dh_top,
                              const void *const *dhT, const void *const *dcT, void *dx_all, void *const *dh0,
                              void *const *dc0, void *const *dVx, void *const *dUx, void *const *dVh, void *const *dUh,
                              void *const *dbias, int accumulate, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    StackGeom g;
    int st = check_stack_desc(d, &g);
    if (st != PF_OK) return st;
    if (!h0 || !c0 || !h_all || !c_all || !gates_all || !Tx_all || !Th_all || !Vx || !Ux || !Vh || !Uh || !dh0 || !dc0 ||
        !dVx || !dUx || !dVh || !dUh)
        return PF_ERR_NULL;
    StackPtrs p = {};
    StackBwdPtrs b = {};
    hipStream_t s = (hipStream_t)stream;
    const int L = g.L, h = g.h, r = g.r, gr = g.gr, B = g.B, T = g.T;
    for (int l = 0; l < L; ++l) {
        if (!Vx[l] || !Ux[l] || !Vh[l] || !Uh[l] || !dVx[l] || !dUx[l] || !dVh[l] || !dUh[l]) return PF_ERR_NULL;
        if (T > 0 && B > 0 &&
            (!h0[l] || !c0[l] || !h_all[l] || !c_all[l] || !gates_all[l] || !Tx_all[l] || !Th_all[l] || !dh0[l] || !dc0[l]))
            return PF_ERR_NULL;
        if (any_misaligned({h0[l], c0[l], h_all[l], c_all[l], gates_all[l], Tx_all[l], Th_all[l], Vx[l], Ux[l], Vh[l], Uh[l],
                            dhT ? dhT[l] : nullptr, dcT ? dcT[l] : nullptr, dh0[l], dc0[l]},
                           16) ||
            any_misaligned({dVx[l], dUx[l], dVh[l], dUh[l], dbias ? dbias[l] : nullptr}, 4))
            return PF_ERR_UNSUPPORTED;
        p.h0[l] = (const float *)h0[l];
        p.c0[l] = (const float *)c0[l];
        p.h_all[l] = (float *)h_all[l];
        p.c_all[l] = (float *)c_all[l];
        p.gates_all[l] = (float *)gates_all[l];
        p.Tx_all[l] = (float *)Tx_all[l];
        p.Th_all[l] = (float *)Th_all[l];
        p.Vx[l] = (const float *)Vx[l];
        p.Ux[l] = (const float *)Ux[l];
        p.Vh[l] = (const float *)Vh[l];
        p.Uh[l] = (const float *)Uh[l];
        b.dhT[l] = dhT ? (const float *)dhT[l] : nullptr;
        b.dcT[l] = dcT ? (const float *)dcT[l] : nullptr;
        b.dh0[l] = (float *)dh0[l];
        b.dc0[l] = (float *)dc0[l];
        b.dVx[l] = (float *)dVx[l];
        b.dUx[l] = (float *)dUx[l];
        b.dVh[l] = (float *)dVh[l];
        b.dUh[l] = (float *)dUh[l];
        b.dbias[l] = dbias ? (float *)dbias[l] : nullptr;
    }
    if (T == 0 || B == 0) { // no rows: the gradients this call owns are zero
        for (int l = 0; l < L && st == PF_OK && !accumulate; ++l) {
            const i64 din = l ? h : g.din;
            st = launch_zero_f32(s, b.dVx[l], din * gr);
            if (st == PF_OK) st = launch_zero_f32(s, b.dVh[l], (i64)h * gr);
            if (st == PF_OK) st = launch_zero_f32(s, b.dUx[l], 4 * (i64)h * r);
            if (st == PF_OK) st = launch_zero_f32(s, b.dUh[l], 4 * (i64)h * r);
            if (st == PF_OK) st = launch_zero_f32(s, b.dbias[l], 4 * (i64)h);
        }
        return st;
    }
    if (!x || !dh_top) return PF_ERR_NULL;
    if (any_misaligned({x, dh_top, dx_all}, 16)) return PF_ERR_UNSUPPORTED;
    StackPlan pl;
    st = plan_stack(g, &pl);
    if (st != PF_OK) return st;
    if (!workspace || workspace_bytes < pl.bwd_bytes) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    Workspace ws(workspace, workspace_bytes);
    for (int l = 0; l < L; ++l) {
        b.dz_all[l] = ws.take<float>(pl.n_dz);
        b.dTh_all[l] = ws.take<float>(pl.n_dT);
        b.dTx_all[l] = ws.take<float>(pl.n_dT);
    }
    float *part = ws.take<float>(pl.n_part);
    float *part2 = ws.take<float>(pl.n_part2);
    float *packed = ws.take<float>(pl.n_pack_b);
    if (!ws.ok()) return PF_ERR_WORKSPACE;
    StackPacked pk = {};
    stack_pack(g, p, true, packed, &pk, false, s, &st);
    if (st != PF_OK) return st;
    StackCarry carry = {};
    for (int u = 0; u < T + L - 1 + (pk.fused_z ? 1 : 0) && st == PF_OK; ++u) // fused: one more slot for the first layer's dh0
        st = stack_bwd_slot(g, p, pk, b, (const float *)dh_top, u, part, pl.n_part, part2, pl.n_part2, carry, false, s,
                            nullptr, nullptr);
    if (st != PF_OK) return st;
    // the input path of the first layer for all steps at once
    const i64 Mt = (i64)T * B;
    if (g.G == 1) {
        st = st_tall(s, "lstm_stack_dTx0=dz*Ux", false, Mt, b.dz_all[0], 4 * (i64)h, p.Ux[0], r, 4 * h, r, b.dTx_all[0], gr,
                     nullptr, part);
    } else {
        for (int q = 0; q < 4 && st == PF_OK; ++q)
            st = st_tall(s, "lstm_stack_dTx0=dz*Ux", false, Mt, b.dz_all[0] + (i64)q * h, 4 * (i64)h,
                         p.Ux[0] + (i64)q * h * r, r, h, r, b.dTx_all[0] + (i64)q * r, gr, nullptr, part);
    }
    if (st != PF_OK) return st;
    if (dx_all) {
        st = st_tall(s, "lstm_stack_dx=dTx*Vxt", true, Mt, b.dTx_all[0], gr, p.Vx[0], gr, gr, g.din, (float *)dx_all, g.din,
                     nullptr, part);
        if (st != PF_OK) return st;
    }
    // parameter gradients, layer by layer, each a few rank-(T B) updates in one launch
    const SliceSumArgs none = {};
    for (int l = 0; l < L && st == PF_OK; ++l) {
        const float *xin = l ? p.h_all[l - 1] : (const float *)x;
        const int din = l ? h : g.din;
        if (Mt >= ST_RANK_MMA_ROWS) {
            // enough rows for the matrix unit; the bias gradient rides on the input path's dU
            RankMmaArgs rm = {};
            rm.accumulate = accumulate;
            bool ok = true;
            for (int path = 0; path < 2; ++path) {
                const float *Tm = path ? p.Th_all[l] : p.Tx_all[l];
                float *dU = path ? b.dUh[l] : b.dUx[l];
                for (int q = 0; q < g.G; ++q)
                    ok = ok && rank_mma_add(rm, nullptr, 0, b.dz_all[l] + (i64)q * h, 4 * (i64)h, Tm + (i64)q * r, gr,
                                            dU + (i64)q * h * r, r, g.G == 1 ? 4 * h : h, r, (int)Mt,
                                            path == 0 && b.dbias[l] ? b.dbias[l] + (i64)q * h : nullptr);
            }
            ok = ok && rank_mma_add(rm, nullptr, 0, xin, din, b.dTx_all[l], gr, b.dVx[l], gr, din, gr, (int)Mt);
            // dVh = sum_t h_{t-1}^T dTh_t: the left operand is h0, then h_0 .. h_{T-2}
            ok = ok && rank_mma_add(rm, p.h0[l], B, p.h_all[l], h, b.dTh_all[l], gr, b.dVh[l], gr, h, gr, (int)Mt);
            if (ok) {
                st = launch_rank_mma(s, "lstm_stack_grads", rm);
                continue;
            }
            // (a dimension below four: the general kernel below takes the layer)
        }
        RankArgs ra = {};
        ra.M = (int)Mt;
        ra.accumulate = accumulate;
        for (int path = 0; path < 2; ++path) {
            const float *Tm = path ? p.Th_all[l] : p.Tx_all[l];
            float *dU = path ? b.dUh[l] : b.dUx[l];
            if (g.G == 1) {
                rank_add(ra, b.dz_all[l], 4 * (i64)h, Tm, gr, dU, r, 4 * h, r);
            } else {
                for (int q = 0; q < 4; ++q)
                    rank_add(ra, b.dz_all[l] + (i64)q * h, 4 * (i64)h, Tm + (i64)q * r, gr, dU + (i64)q * h * r, r, h, r);
            }
        }
        rank_add(ra, xin, din, b.dTx_all[l], gr, b.dVx[l], gr, din, gr);
        // dVh = sum_t h_{t-1}^T dTh_t: the rows t >= 1 here, the h0 row block in a second launch below
        if (T > 1) rank_add(ra, p.h_all[l], h, b.dTh_all[l] + (i64)B * gr, gr, b.dVh[l], gr, h, gr, (int)(Mt - B));
        if (b.dbias[l]) rank_add(ra, b.dz_all[l], 4 * (i64)h, nullptr, 0, b.dbias[l], 1, 4 * h, 1);
        st = launch_rank_update(s, "lstm_stack_grads", ra, none);
        if (st != PF_OK) return st;
        RankArgs rb = {};
        rb.M = B;
        rb.accumulate = (T > 1) ? 1 : accumulate;
        rank_add(rb, p.h0[l], h, b.dTh_all[l], gr, b.dVh[l], gr, h, gr);
        st = launch_rank_update(s, "lstm_stack_grads", rb, none);
    }
    return st;
}

// ---- one layer over a sequence: a stack of one layer ----
static pf_lstm_stack_desc seq_as_stack(const pf_lstm_seq_desc *d)
{
    pf_lstm_stack_desc sd = {};
    if (d) {
        sd.T = d->T;
        sd.B = d->B;
        sd.d_in = d->d_in;
        sd.h = d->h;
        sd.r = d->r;
        sd.groups = d->groups;
        sd.layers = 1;
        sd.dtype = d->dtype;
        sd.has_bias = d->has_bias;
    }
    return sd;
}

size_t pf_lowrank_lstm_seq_fwd_workspace_bytes(const pf_lstm_seq_desc *d)
{
    if (!d) return 0;
    const pf_lstm_stack_desc sd = seq_as_stack(d);
    return pf_lowrank_lstm_stack_fwd_workspace_bytes(&sd);
}

size_t pf_lowrank_lstm_seq_bwd_workspace_bytes(const pf_lstm_seq_desc *d)
{
    if (!d) return 0;
    const pf_lstm_stack_desc sd = seq_as_stack(d);
    return pf_lowrank_lstm_stack_bwd_workspace_bytes(&sd);
}

int pf_lowrank_lstm_seq_fwd(const pf_lstm_seq_desc *d, const void *x, const void *h0, const void *c0, const void *Vx,
                            const void *Ux, const void *Vh, const void *Uh, const void *bias, void *h_all, void *c_all,
                            void *gates_all, void *Tx_all, void *Th_all, void *workspace, size_t workspace_bytes,
                            void *stream)
{
    if (!d) return PF_ERR_NULL;
    const pf_lstm_stack_desc sd = seq_as_stack(d);
    return pf_lowrank_lstm_stack_fwd(&sd, x, &h0, &c0, &Vx, &Ux, &Vh, &Uh, &bias, &h_all, &c_all, &gates_all, &Tx_all,
                                     &Th_all, workspace, workspace_bytes, stream);
}

int pf_lowrank_lstm_seq_bwd(const pf_lstm_seq_desc *d, const void *x, const void *h0, const void *c0, const void *h_all,
                            const void *c_all, const void *gates_all, const void *Tx_all, const void *Th_all,
                            const void *Vx, const void *Ux, const void *Vh, const void *Uh, const void *dh_all,
                            const void *dhT, const void *dcT, void *dx_all, void *dh0, void *dc0, void *dVx, void *dUx,
                            void *dVh, void *dUh, void *dbias, int accumulate, void *workspace, size_t workspace_bytes,
                            void *stream)
{
    if (!d) return PF_ERR_NULL;
    const pf_lstm_stack_desc sd = seq_as_stack(d);
    return pf_lowrank_lstm_stack_bwd(&sd, x, &h0, &c0, &h_all, &c_all, &gates_all, &Tx_all, &Th_all, &Vx, &Ux, &Vh, &Uh,
                                     dh_all, &dhT, &dcT, dx_all, &dh0, &dc0, &dVx, &dUx, &dVh, &dUh, &dbias, accumulate,
                                     workspace, workspace_bytes, stream);
}

} // extern "C"
