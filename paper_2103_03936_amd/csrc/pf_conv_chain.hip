// Fused two-stage convolution chain kernel (see pf_conv_chain.h) and its weight packers.
#include "pf_conv_chain.h"

namespace pf {

constexpr int CH_PIX = 64;           // pixel slots of one image tile
constexpr int CH_PP = 101;           // padded positions (up to 10 x 10) plus one all-zero row
constexpr int CH_SUB = 64;           // channels staged per wavefront at a time
constexpr int CH_XLD = CH_SUB + 8;   // row stride (elements) of the staged input tile: 144 bytes
constexpr int CH_PLD = CH_PIX + 1;   // row stride (floats) of a partial-sum tile

typedef uint4 __attribute__((may_alias)) uint4_alias;

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

template <int KS1, int KS2, int R>
__global__ __launch_bounds__(256, 1) void conv_chain_kernel(ChainArgs a)
{
    constexpr int RB = R / 32, T1 = KS1 * KS1, T2 = KS2 * KS2;
    constexpr int TLD = R + 8; // row stride (elements) of the intermediate tile
    constexpr int S2 = T2 * (R / 16);
    __shared__ __attribute__((aligned(16))) uint16_t Xs[4][CH_PP * CH_XLD];
    __shared__ __attribute__((aligned(16))) float P[4][64 * CH_PLD];
    __shared__ __attribute__((aligned(16))) uint16_t Ts[CH_PP * TLD];
    __shared__ uint16_t pp1[CH_PIX], pp2[CH_PIX];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int n = blockIdx.x;
    const int H = a.H, W = a.W, HW = H * W, C1 = a.C1, C2 = a.C2;
    const int Wp1 = KS1 == 3 ? W + 2 : W, Wp2 = KS2 == 3 ? W + 2 : W;
    const int Z1 = KS1 == 3 ? (H + 2) * (W + 2) : HW; // index of the all-zero row
    const int Z2 = KS2 == 3 ? (H + 2) * (W + 2) : HW;

    // ---- set-up: pixel -> padded-position tables, zero the tiles (borders stay zero) ----
    if (tid < CH_PIX) {
        const int y = tid / W, x = tid - y * W;
        pp1[tid] = (uint16_t)(tid < HW ? (KS1 == 3 ? (y + 1) * Wp1 + x + 1 : tid) : Z1);
        pp2[tid] = (uint16_t)(tid < HW ? (KS2 == 3 ? (y + 1) * Wp2 + x + 1 : tid) : Z2);
    }
    {
        uint4 z = make_uint4(0, 0, 0, 0);
        uint4_alias *x4 = (uint4_alias *)&Xs[0][0];
        for (int i = tid; i < 4 * CH_PP * CH_XLD / 8; i += 256) x4[i] = z;
        uint4_alias *t4 = (uint4_alias *)&Ts[0];
        for (int i = tid; i < CH_PP * TLD / 8; i += 256) t4[i] = z;
    }
    __syncthreads();

    // top-left padded position of this lane's two pixels (pixel blocks 0 and 1)
    int pos1[2], pos2[2];
    bool valid[2];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        const int p = 32 * pb + col;
        valid[pb] = p < HW;
        pos1[pb] = valid[pb] ? pp1[p] - (KS1 == 3 ? Wp1 + 1 : 0) : Z1;
        pos2[pb] = valid[pb] ? pp2[p] - (KS2 == 3 ? Wp2 + 1 : 0) : Z2;
    }

    // ------------------------------- stage 1 -------------------------------
    f32x16_t acc[RB][2];
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][pb][v] = 0.f;

    uint16_t *xs = &Xs[w][0];
    const int cw = C1 / 4;        // channels of this wavefront
    const int nsub = cw / CH_SUB; // staging rounds
    const int nvec = CH_SUB * HW / 8;
    for (int sub = 0; sub < nsub; ++sub) {
        const int cb = w * cw + sub * CH_SUB;
        // stage channels [cb, cb + 64) of image n, transposed to [padded position][channel]
        if (sub > 0) __syncthreads(); // the previous round's fragment reads are done
        const uint4 *src = (const uint4 *)(a.in + ((i64)n * C1 + cb) * HW);
        for (int vi = lane; vi < nvec; vi += 64) {
            const uint4 d = src[vi];
            int c = (8 * vi) / HW, p = 8 * vi - c * HW;
            const uint32_t dw[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                xs[pp1[p] * CH_XLD + c] = (uint16_t)(dw[e >> 1] >> (16 * (e & 1)));
                if (++p == HW) {
                    p = 0;
                    ++c;
                }
            }
        }
        __syncthreads();
#pragma unroll 1
        for (int c16 = 0; c16 < CH_SUB / 16; ++c16) {
            const i64 s0 = (i64)((cb >> 4) + c16) * T1;
            uint4 af[T1][RB];
#pragma unroll
            for (int t = 0; t < T1; ++t)
#pragma unroll
                for (int b = 0; b < RB; ++b) af[t][b] = a.W1p[((s0 + t) * RB + b) * 64 + lane];
#pragma unroll
            for (int t = 0; t < T1; ++t) {
                const int toff = KS1 == 3 ? (t / 3) * Wp1 + (t % 3) : 0;
                bf16x8_t bfr[2];
#pragma unroll
                for (int pb = 0; pb < 2; ++pb)
                    bfr[pb] = as_bf16x8(lds_read16(&xs[(pos1[pb] + (valid[pb] ? toff : 0)) * CH_XLD + 16 * c16 + 8 * half]));
#pragma unroll
                for (int b = 0; b < RB; ++b)
#pragma unroll
                    for (int pb = 0; pb < 2; ++pb)
                        acc[b][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(af[t][b]), bfr[pb], acc[b][pb], 0, 0, 0);
            }
        }
    }

    // ---------------- sum the four partial tiles, 64 rows of rho at a time ----------------
#pragma unroll
    for (int rh = 0; rh < R / 64; ++rh) {
        if (rh > 0) __syncthreads();
        float *pw = &P[w][0];
#pragma unroll
        for (int bb = 0; bb < 2; ++bb)
#pragma unroll
            for (int pb = 0; pb < 2; ++pb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    pw[(32 * bb + 8 * (v >> 2) + 4 * half + (v & 3)) * CH_PLD + 32 * pb + col] = acc[2 * rh + bb][pb][v];
        __syncthreads();
        const int pix = tid & 63;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int r0 = 8 * ((tid >> 6) + 4 * it);
            uint16_t o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int idx = (r0 + e) * CH_PLD + pix;
                o[e] = float_to_bf16_bits((P[0][idx] + P[1][idx]) + (P[2][idx] + P[3][idx]));
            }
            if (pix < HW) {
                uint4 pk;
                pk.x = o[0] | ((uint32_t)o[1] << 16);
                pk.y = o[2] | ((uint32_t)o[3] << 16);
                pk.z = o[4] | ((uint32_t)o[5] << 16);
                pk.w = o[6] | ((uint32_t)o[7] << 16);
                *(uint4_alias *)&Ts[pp2[pix] * TLD + 64 * rh + r0] = pk;
                if (a.mid_save) {
                    uint16_t *ms = a.mid_save + ((i64)n * R + 64 * rh + r0) * HW + pix;
#pragma unroll
                    for (int e = 0; e < 8; ++e) ms[(i64)e * HW] = o[e];
                }
            }
        }
    }
    __syncthreads();

    // ------------------------------- stage 2 -------------------------------
    const int nb2 = C2 / 32;
    for (int ob = 2 * w; ob < nb2; ob += 8) {
        f32x16_t acc2[2][2];
#pragma unroll
        for (int bb = 0; bb < 2; ++bb)
#pragma unroll
            for (int pb = 0; pb < 2; ++pb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc2[bb][pb][v] = 0.f;
        const uint4 *w2a = a.W2p + ((i64)ob * S2) * 64 + lane;
        const uint4 *w2b = w2a + (i64)S2 * 64;
#pragma unroll
        for (int t = 0; t < T2; ++t) {
            const int toff = KS2 == 3 ? (t / 3) * Wp2 + (t % 3) : 0;
#pragma unroll
            for (int r16 = 0; r16 < R / 16; ++r16) {
                const int s2 = t * (R / 16) + r16;
                const uint4 a0 = w2a[s2 * 64], a1 = w2b[s2 * 64];
                bf16x8_t bfr[2];
#pragma unroll
                for (int pb = 0; pb < 2; ++pb)
                    bfr[pb] = as_bf16x8(lds_read16(&Ts[(pos2[pb] + (valid[pb] ? toff : 0)) * TLD + 16 * r16 + 8 * half]));
#pragma unroll
                for (int pb = 0; pb < 2; ++pb) {
                    acc2[0][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a0), bfr[pb], acc2[0][pb], 0, 0, 0);
                    acc2[1][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a1), bfr[pb], acc2[1][pb], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int bb = 0; bb < 2; ++bb)
#pragma unroll
            for (int pb = 0; pb < 2; ++pb) {
                const int pix = 32 * pb + col;
                if (pix < HW) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int o = 32 * (ob + bb) + 8 * (v >> 2) + 4 * half + (v & 3);
                        a.out[((i64)n * C2 + o) * HW + pix] = float_to_bf16_bits(acc2[bb][pb][v]);
                    }
                }
            }
    }
}

// ------------------------------------------------------------------ packers
__global__ __launch_bounds__(256) void pack_chain_w1_kernel(const uint16_t *src, uint4 *dst, int nfrag_lanes, int RB,
                                                             int T, i64 s_rho, i64 s_c, i64 s_tap)
{
    const int g = blockIdx.x * 256 + threadIdx.x; // one 16-byte fragment slot: ((s * RB + b) * 64 + lane)
    if (g >= nfrag_lanes) return;
    const int lane = g & 63, fb = g >> 6, b = fb % RB, s = fb / RB;
    const int rho = 32 * b + (lane & 31), c0 = 16 * (s / T) + 8 * (lane >> 5), tap = s % T;
    uint16_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = src[rho * s_rho + (c0 + i) * s_c + tap * s_tap];
    uint4 pk;
    pk.x = e[0] | ((uint32_t)e[1] << 16);
    pk.y = e[2] | ((uint32_t)e[3] << 16);
    pk.z = e[4] | ((uint32_t)e[5] << 16);
    pk.w = e[6] | ((uint32_t)e[7] << 16);
    dst[g] = pk;
}

__global__ __launch_bounds__(256) void pack_chain_w2_kernel(const uint16_t *src, uint4 *dst, int nfrag_lanes, int S2,
                                                             int R16, i64 base, i64 s_o, i64 s_rho, i64 s_tap)
{
    const int g = blockIdx.x * 256 + threadIdx.x; // ((ob * S2 + s2) * 64 + lane)
    if (g >= nfrag_lanes) return;
    const int lane = g & 63, fb = g >> 6, s2 = fb % S2, ob = fb / S2;
    const int o = 32 * ob + (lane & 31), tap = s2 / R16, rho0 = 16 * (s2 % R16) + 8 * (lane >> 5);
    uint16_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = src[base + o * s_o + (rho0 + i) * s_rho + tap * s_tap];
    uint4 pk;
    pk.x = e[0] | ((uint32_t)e[1] << 16);
    pk.y = e[2] | ((uint32_t)e[3] << 16);
    pk.z = e[4] | ((uint32_t)e[5] << 16);
    pk.w = e[6] | ((uint32_t)e[7] << 16);
    dst[g] = pk;
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

int launch_pack_chain_w1(hipStream_t s, const uint16_t *src, uint4 *dst, int C1, int R, int k, i64 s_rho, i64 s_c,
                         i64 s_tap)
{
    int st = PF_OK;
    const int T = k * k, RB = R / 32;
    const int n = T * (C1 / 16) * RB * 64;
    PF_LAUNCH(st, "pack_chain_w1", pack_chain_w1_kernel, dim3((n + 255) / 256), dim3(256), s, src, dst, n, RB, T, s_rho,
              s_c, s_tap);
    return st;
}

int launch_pack_chain_w2(hipStream_t s, const uint16_t *src, uint4 *dst, int C2, int R, int k, i64 base, i64 s_o,
                         i64 s_rho, i64 s_tap)
{
    int st = PF_OK;
    const int S2 = k * k * (R / 16);
    const int n = (C2 / 32) * S2 * 64;
    PF_LAUNCH(st, "pack_chain_w2", pack_chain_w2_kernel, dim3((n + 255) / 256), dim3(256), s, src, dst, n, S2, R / 16,
              base, s_o, s_rho, s_tap);
    return st;
}

int launch_conv_chain(hipStream_t s, const char *name, const ChainArgs &a, int N, int k1, int k2, int R)
{
    int st = PF_OK;
    if (N <= 0) return st;
    const dim3 grid(N), block(256);
#define PF_CHAIN_CASE(K1, K2, RR)                                                                   \
    if (k1 == K1 && k2 == K2 && R == RR) {                                                          \
        PF_LAUNCH(st, name, (conv_chain_kernel<K1, K2, RR>), grid, block, s, a);                    \
        return st;                                                                                  \
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
