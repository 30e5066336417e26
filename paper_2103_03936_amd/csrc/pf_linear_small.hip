// Factorized linear layer in fp32 for a small batch (M <= 128 rows; the fully connected layers of a CNN head,
// Section 2.1): two launches per direction.
//
// At these sizes one product has too little work for the chip unless the long contraction (in or out, hundreds)
// is cut into slices, and every slice needs its own compute unit: the fp32 matrix instruction gives one compute
// unit 0.6 TFLOP/s.  So
//   launch 1 (ls_slices_kernel):   P[s] = X[:, slice s] V[slice s, :]   (32 x 32 tiles x S slices of the contraction)
//   launch 2 (ls_tiles_kernel):    every tile of every product that reads T = sum_s P[s]:  Y = T U^T + b forward;
//                                  dX = dT V^T, dU = dY^T T, dV = X^T dT, db backward (dT from its slices)
// and the slice sum is taken where an operand is staged in LDS, not by a launch of its own.  The rank-r intermediate
// crosses launches as S slices of M x r floats that stay in the last-level cache.
#include "pf_linear_small.h"

namespace pf {

constexpr int LS_PITCH = 33; // floats between the k rows of a staged operand tile (32 values + 1 against conflicts)

// ----------------------------------------------------------------- launch 1
// P[s][m][n] = sum over k in slice s of A[m][k] W[k][n]; grid (N / 32, row blocks, S).  The four wavefronts take a
// quarter of the slice each and add their tiles in LDS.
__global__ __launch_bounds__(256) void ls_slices_kernel(LsSliceArgs a0, LsSliceArgs a1)
{
    const LsSliceArgs a = blockIdx.z >= (unsigned)a0.S ? a1 : a0;
    const int s = blockIdx.z >= (unsigned)a0.S ? blockIdx.z - a0.S : blockIdx.z;
    const int ct = blockIdx.x, rb = blockIdx.y;
    if (ct * 32 >= a.N) return; // (the two problems may differ in width)
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, col = lane & 31;
    const int KS = a.K / a.S, kq = KS / 4; // kq: a multiple of 8
    const int k0 = s * KS + w * kq;
    const int row = rb * 32 + col;
    const float *Ar = a.A + (i64)(row < a.M ? row : a.M - 1) * a.lda;
    const float *Wc = a.W + ct * 32 + col;
    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int kb = 0; kb < kq; kb += 8) { // lane half h holds k = k0 + kb + 4 h + 0..3
        const int k = k0 + kb + 4 * half;
        f32x4_t av = *(const f32x4_t *)(Ar + k);
        if (row >= a.M) av = f32x4_t{0.f, 0.f, 0.f, 0.f};
        float bv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[j] = Wc[(i64)(k + j) * a.ldw];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[j], bv[j], acc, 0, 0, 0);
    }
    __shared__ float red[4][32 * LS_PITCH];
#pragma unroll
    for (int v = 0; v < 16; ++v) red[w][(8 * (v >> 2) + 4 * half + (v & 3)) * LS_PITCH + col] = acc[v];
    __syncthreads();
    float *P = a.P + (i64)s * a.M * a.N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = tid + 256 * i, m = e >> 5, n = e & 31;
        const float v = (red[0][m * LS_PITCH + n] + red[1][m * LS_PITCH + n]) + (red[2][m * LS_PITCH + n] + red[3][m * LS_PITCH + n]);
        if (rb * 32 + m < a.M) P[(i64)(rb * 32 + m) * a.N + ct * 32 + n] = v;
    }
}

// ----------------------------------------------------------------- launch 2
// One 32 x 32 output tile per workgroup: C[m][n] = sum_k A(m, k) B(k, n), k < K <= LS_MAX_K.  Both operands are
// staged in LDS k-major (element (k, i) at k * 33 + i), read from memory along their fast index:
//   LS_MK: element (i, k) at p[i * ld + k]   (a row-major activation, or U / V read as the right operand)
//   LS_KM: element (i, k) at p[k * ld + i]   (dY or X as the left operand of a factor gradient; T as the right one)
// and either may be the sum of `slices` slices `sstride` floats apart.
// (16-byte loads along the fast index; the loads of all slices of a piece are issued before the first add, and
// slices are added in order)
// SL: whether the operand comes in slices.  The loads are unconditional (a slice index past the end re-reads slice
// 0 and is left out of the sum), so that all of them are in flight together.
template <bool SL>
__device__ __forceinline__ f32x4_t ls_piece(const float *p, int slices, i64 sstride, bool live)
{
    if (!SL) {
        const f32x4_t v = *(const f32x4_t *)p;
        return live ? v : f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    f32x4_t v[LS_MAX_SLICES];
#pragma unroll
    for (int sl = 0; sl < LS_MAX_SLICES; ++sl) v[sl] = *(const f32x4_t *)(p + (i64)(sl < slices ? sl : 0) * sstride);
    f32x4_t sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int sl = 0; sl < LS_MAX_SLICES; ++sl) {
        const float keep = sl < slices ? 1.f : 0.f;
        sum += v[sl] * keep;
    }
    return live ? sum : f32x4_t{0.f, 0.f, 0.f, 0.f};
}

template <bool SL>
__device__ __forceinline__ void ls_stage(float *dst, const LsOperand &o, int i0, int ni, int K, int tid)
{
    if (o.layout == LS_MK) { // piece = 4 consecutive k of row i (K a multiple of 4); consecutive threads along k
        const int k4n = K >> 2, total = 32 * k4n;
#pragma unroll 4
        for (int e = tid; e < total; e += 256) {
            const int i = e / k4n, k = 4 * (e - i * k4n);
            const bool live = i0 + i < ni;
            const f32x4_t v = ls_piece<SL>(o.p + (i64)(live ? i0 + i : i0) * o.ld + k, o.slices, o.sstride, live);
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[(k + j) * LS_PITCH + i] = v[j];
        }
    } else { // piece = 4 consecutive i of row k; consecutive threads along i
        const int total = 8 * K;
#pragma unroll 4
        for (int e = tid; e < total; e += 256) {
            const int k = e >> 3, i = 4 * (e & 7);
            const bool live = i0 + i < ni; // (ni is a multiple of 4 wherever this layout is used)
            const f32x4_t v = ls_piece<SL>(o.p + (i64)k * o.ld + (live ? i0 + i : i0), o.slices, o.sstride, live);
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[k * LS_PITCH + i + j] = v[j];
        }
    }
}

__global__ __launch_bounds__(256) void ls_tiles_kernel(LsTileArgs a)
{
    // which problem does this workgroup belong to?
    int q = 0;
#pragma unroll
    for (int i = 1; i < LS_MAX_PROB; ++i)
        if (i < a.nprob && (int)blockIdx.x >= a.p[i].wg0) q = i;
    const LsTileProb &pr = a.p[q];
    const int t = blockIdx.x - pr.wg0, nt = (pr.N + 31) / 32;
    const int m0 = 32 * (t / nt), n0 = 32 * (t % nt);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, col = lane & 31;
    __shared__ float As[LS_MAX_K * LS_PITCH], Bs[LS_MAX_K * LS_PITCH];
    __shared__ float red[4][32 * LS_PITCH];
    const int K = pr.K;
    if (pr.A.slices > 1) // (uniform)
        ls_stage<true>(As, pr.A, m0, pr.M, K, tid);
    else
        ls_stage<false>(As, pr.A, m0, pr.M, K, tid);
    if (pr.B.slices > 1)
        ls_stage<true>(Bs, pr.B, n0, pr.N, K, tid);
    else
        ls_stage<false>(Bs, pr.B, n0, pr.N, K, tid);
    __syncthreads();
    if (pr.A_copy && n0 == 0) { // the summed left operand leaves once (T for the backward pass): [M][K]
        for (int e = tid; e < 32 * K; e += 256) {
            const int i = e / K, k = e - i * K;
            if (m0 + i < pr.M) pr.A_copy[(i64)(m0 + i) * K + k] = As[k * LS_PITCH + i];
        }
    }
    if (pr.colsum && n0 == 0 && tid < 32 && m0 + tid < pr.M) { // sum of the left operand over k (a bias gradient)
        float part[4] = {0.f, 0.f, 0.f, 0.f}; // four running sums: the LDS reads do not wait for one another
        for (int k = 0; k < K; k += 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) part[j] += k + j < K ? As[(k + j) * LS_PITCH + tid] : 0.f;
        }
        const float sum = (part[0] + part[1]) + (part[2] + part[3]);
        pr.colsum[m0 + tid] = pr.accumulate ? pr.colsum[m0 + tid] + sum : sum;
    }
    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    // wavefront w takes k = 2 (4 j + w) + half: the k pairs are dealt round the four wavefronts
    for (int kp = w; 2 * kp < K; kp += 16) { // four k pairs per round: their LDS reads go out together
        float av[4], bv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = 2 * (kp + 4 * u) + half;
            av[u] = k < K ? As[k * LS_PITCH + col] : 0.f;
            bv[u] = k < K ? Bs[k * LS_PITCH + col] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[u], acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) red[w][(8 * (v >> 2) + 4 * half + (v & 3)) * LS_PITCH + col] = acc[v];
    __syncthreads();
    if (!pr.C) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = tid + 256 * i, m = e >> 5, n = e & 31;
        if (m0 + m < pr.M && n0 + n < pr.N) {
            float v = (red[0][m * LS_PITCH + n] + red[1][m * LS_PITCH + n]) + (red[2][m * LS_PITCH + n] + red[3][m * LS_PITCH + n]);
            if (pr.bias) v += pr.bias[n0 + n];
            float *c = pr.C + (i64)(m0 + m) * pr.ldc + n0 + n;
            *c = pr.accumulate ? *c + v : v;
        }
    }
}

bool linear_small_supported(i64 M, i64 n_in, i64 n_out, i64 r)
{
    return M > 0 && M <= LS_MAX_K && r <= LS_MAX_K && n_in % 32 == 0 && n_out % 32 == 0 && r % 32 == 0 && n_in >= 32 &&
           n_out >= 32 && r >= 32 && n_in <= (1 << 20) && n_out <= (1 << 20);
}

int linear_small_slices(i64 K)
{
    for (int s = 8; s > 1; s >>= 1)
        if (K % (32 * s) == 0) return s;
    return 1;
}

int launch_ls_slices(hipStream_t s, const char *name, const LsSliceArgs &a0, const LsSliceArgs &a1)
{
    int st = PF_OK;
    const int n = a0.N > a1.N ? a0.N : a1.N, m = a0.M > a1.M ? a0.M : a1.M;
    if (n <= 0 || m <= 0) return st;
    const dim3 grid((unsigned)(n / 32), (unsigned)((m + 31) / 32), (unsigned)(a0.S + a1.S));
    PF_LAUNCH(st, name, ls_slices_kernel, grid, dim3(256), s, a0, a1);
    return st;
}

void ls_add(LsTileArgs &a, const LsOperand &A, const LsOperand &B, int M, int N, int K, float *C, i64 ldc, const float *bias,
            int accumulate, float *A_copy, float *colsum)
{
    LsTileProb &p = a.p[a.nprob++];
    p.A = A;
    p.B = B;
    p.M = M;
    p.N = N;
    p.K = K;
    p.C = C;
    p.ldc = ldc;
    p.bias = bias;
    p.accumulate = accumulate;
    p.A_copy = A_copy;
    p.colsum = colsum;
    p.wg0 = a.nwg;
    a.nwg += ((M + 31) / 32) * ((N + 31) / 32);
}

int launch_ls_tiles(hipStream_t s, const char *name, const LsTileArgs &a)
{
    int st = PF_OK;
    if (a.nwg <= 0) return st;
    PF_LAUNCH(st, name, ls_tiles_kernel, dim3((unsigned)a.nwg), dim3(256), s, a);
    return st;
}

} // namespace pf
