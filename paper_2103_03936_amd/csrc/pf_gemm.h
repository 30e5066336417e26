// Guarded MFMA tile GEMM with functor operands: C(m,n) = sum_k A(m,k) B(k,n).
//
// One workgroup (4 wavefronts) owns a 64 x 64 tile of C; each wavefront owns a
// 32 x 32 block and feeds one 32x32 MFMA per k-step from LDS.  Operands are
// fetched element by element through functors, so any shape, transposition or
// im2col view works; out-of-range elements read as zero.  This is the
// any-shape path; aligned shapes take the vectorised kernels elsewhere.
//
// LDS tiles are [row][k] with k contiguous.  A lane's fragment is 16 bytes:
//   bf16: 8 values k = 16 kk + 8 (lane / 32) + 0..7  -> one 32x32x16 MFMA
//   f32 : 4 values k =  8 kk + 4 (lane / 32) + 0..3  -> four 32x32x2 MFMAs, the q-th of
//         which takes element q from both halves of the wavefront (A and B agree on
//         which k that is, which is all the instruction needs).
// Accumulator element v of lane l is C(8 (v / 4) + 4 (l / 32) + v % 4, l % 32).
#pragma once

#include "pf_common.h"

namespace pf {

constexpr int GEMM_BM = 64, GEMM_BN = 64, GEMM_BK = 32;

template <typename CT>
struct LdsTraits;
template <>
struct LdsTraits<float> {
    typedef float elem;
    static constexpr int LDK = GEMM_BK + 4; // 144-byte rows
    static __device__ __forceinline__ elem cvt(float f) { return f; }
};
template <>
struct LdsTraits<bf16_t> {
    typedef uint16_t elem;
    static constexpr int LDK = GEMM_BK + 8; // 80-byte rows
    static __device__ __forceinline__ elem cvt(float f) { return float_to_bf16_bits(f); }
};

// acc += A_block(32 x 32k) * B_block(32k x 32) from LDS rows of stride LDK.
__device__ __forceinline__ void mma_32x32_k32(f32x16_t &acc, const float *As, const float *Bs, int lane)
{
    constexpr int LDK = LdsTraits<float>::LDK;
    const int row = lane & 31, half = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < GEMM_BK / 8; ++kk) {
        f32x4_t a = *(const f32x4_t *)&As[row * LDK + kk * 8 + half * 4];
        f32x4_t b = *(const f32x4_t *)&Bs[row * LDK + kk * 8 + half * 4];
#pragma unroll
        for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q], b[q], acc, 0, 0, 0);
    }
}

__device__ __forceinline__ void mma_32x32_k32(f32x16_t &acc, const uint16_t *As, const uint16_t *Bs, int lane)
{
    constexpr int LDK = LdsTraits<bf16_t>::LDK;
    const int row = lane & 31, half = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < GEMM_BK / 16; ++kk) {
        bf16x8_t a = *(const bf16x8_t *)&As[row * LDK + kk * 16 + half * 8];
        bf16x8_t b = *(const bf16x8_t *)&Bs[row * LDK + kk * 16 + half * 8];
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
}

// A_KFAST / B_KFAST: whether neighbouring threads should walk k (true) or the row/column
// index (false) when filling the tile -- pick whichever is contiguous in memory.
// blockIdx.z = zb * ksplit + ks: zb is a batch index handed to the functors (gate of an
// LSTM, ...), ks selects the k-range [ks * k_per_split, (ks + 1) * k_per_split).
template <typename CT, bool A_KFAST, bool B_KFAST, typename AF, typename BF, typename EF>
__global__ __launch_bounds__(256) void gemm_generic_kernel(AF af, BF bf, EF ef, int M, int N, int K,
                                                            int ksplit, int k_per_split)
{
    typedef typename LdsTraits<CT>::elem elem;
    constexpr int LDK = LdsTraits<CT>::LDK;
    __shared__ __attribute__((aligned(16))) elem As[GEMM_BM * LDK];
    __shared__ __attribute__((aligned(16))) elem Bs[GEMM_BN * LDK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.x * GEMM_BM, n0 = blockIdx.y * GEMM_BN;
    const int zb = blockIdx.z / ksplit, ks = blockIdx.z % ksplit;
    const int kbeg = ks * k_per_split;
    const int kend = min(K, kbeg + k_per_split);

    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    for (int k0 = kbeg; k0 < kend; k0 += GEMM_BK) {
#pragma unroll
        for (int e = 0; e < GEMM_BM * GEMM_BK / 256; ++e) {
            const int idx = e * 256 + tid;
            const int kk = A_KFAST ? (idx % GEMM_BK) : (idx / GEMM_BM);
            const int mm = A_KFAST ? (idx / GEMM_BK) : (idx % GEMM_BM);
            const int gm = m0 + mm, gk = k0 + kk;
            float v = 0.f;
            if (gm < M && gk < kend) v = af(gm, gk, zb);
            As[mm * LDK + kk] = LdsTraits<CT>::cvt(v);
        }
#pragma unroll
        for (int e = 0; e < GEMM_BN * GEMM_BK / 256; ++e) {
            const int idx = e * 256 + tid;
            const int kk = B_KFAST ? (idx % GEMM_BK) : (idx / GEMM_BN);
            const int nn = B_KFAST ? (idx / GEMM_BK) : (idx % GEMM_BN);
            const int gn = n0 + nn, gk = k0 + kk;
            float v = 0.f;
            if (gn < N && gk < kend) v = bf(gk, gn, zb);
            Bs[nn * LDK + kk] = LdsTraits<CT>::cvt(v);
        }
        __syncthreads();
        if (sizeof(elem) == 4) {
            // float path: sum each 32-deep k-chunk on its own and add it to the running total, so the
            // rounding error grows with the number of chunks rather than with K
            f32x16_t chunk;
#pragma unroll
            for (int v = 0; v < 16; ++v) chunk[v] = 0.f;
            mma_32x32_k32(chunk, &As[wm * 32 * LDK], &Bs[wn * 32 * LDK], lane);
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] += chunk[v];
        } else {
            mma_32x32_k32(acc, &As[wm * 32 * LDK], &Bs[wn * 32 * LDK], lane);
        }
        __syncthreads();
    }

    const int col = lane & 31, half = lane >> 5;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int gm = m0 + wm * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
        const int gn = n0 + wn * 32 + col;
        if (gm < M && gn < N) ef(gm, gn, acc[v], zb, ks);
    }
}

// out[i] (+)= sum_s partial[s * count + i]
__global__ void splitk_reduce_kernel(const float *partial, float *out, i64 count, int ksplit, int accumulate);
// out[i] = 0
__global__ void zero_f32_kernel(float *out, i64 count);

struct GemmShape {
    int M, N, K;
    int batch;  // functor batch count (zb)
    int ksplit; // number of k-ranges
};

template <typename CT, bool A_KFAST, bool B_KFAST, typename AF, typename BF, typename EF>
inline int launch_gemm_generic(const char *name, hipStream_t stream, GemmShape s, AF af, BF bf, EF ef)
{
    int status = PF_OK;
    if (s.M <= 0 || s.N <= 0 || s.batch <= 0) return status;
    const int ksplit = s.ksplit < 1 ? 1 : s.ksplit;
    int k_per = (s.K + ksplit - 1) / ksplit;
    k_per = (k_per + GEMM_BK - 1) / GEMM_BK * GEMM_BK;
    if (k_per < GEMM_BK) k_per = GEMM_BK;
    dim3 grid((s.M + GEMM_BM - 1) / GEMM_BM, (s.N + GEMM_BN - 1) / GEMM_BN, s.batch * ksplit);
    PF_LAUNCH(status, name, (gemm_generic_kernel<CT, A_KFAST, B_KFAST, AF, BF, EF>), grid, dim3(256), stream, af,
              bf, ef, s.M, s.N, s.K, ksplit, k_per);
    return status;
}

// Pick a k-split that gives the machine a few workgroups per compute unit.
inline int choose_ksplit(i64 M, i64 N, i64 K, int batch = 1)
{
    i64 tiles = ((M + GEMM_BM - 1) / GEMM_BM) * ((N + GEMM_BN - 1) / GEMM_BN) * batch;
    if (tiles <= 0) return 1; // empty product
    i64 want = (512 + tiles - 1) / tiles;
    i64 kmax = (K + 4 * GEMM_BK - 1) / (4 * GEMM_BK); // at least 4 k-steps per split
    if (want > kmax) want = kmax;
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    return (int)want;
}

// ---------------------------------------------------------------- functors
// Operand A(m,k) or B(k,n) over a plain matrix.  "Row" means the non-k index.
template <typename T>
struct OpA_RowMajor { // A(m,k) = p[m * ld + zb * zoff + k]
    const T *p;
    i64 ld;
    i64 zoff;
    __device__ __forceinline__ float operator()(int m, int k, int zb) const
    {
        return to_float(p[(i64)m * ld + zb * zoff + k]);
    }
};
template <typename T>
struct OpA_ColMajor { // A(m,k) = p[k * ld + zb * zoff + m]
    const T *p;
    i64 ld;
    i64 zoff;
    __device__ __forceinline__ float operator()(int m, int k, int zb) const
    {
        return to_float(p[(i64)k * ld + zb * zoff + m]);
    }
};
template <typename T>
struct OpB_NK { // B(k,n) = p[(zb * zoff + n) * ld + k]   (matrix stored [N][K])
    const T *p;
    i64 ld;
    i64 zoff;
    __device__ __forceinline__ float operator()(int k, int n, int zb) const
    {
        return to_float(p[(zb * zoff + n) * ld + k]);
    }
};
template <typename T>
struct OpB_KN { // B(k,n) = p[(zb * zrow + k) * ld + zb * zcol + n]   (matrix stored [K][N])
    const T *p;
    i64 ld;
    i64 zrow, zcol;
    __device__ __forceinline__ float operator()(int k, int n, int zb) const
    {
        return to_float(p[(zb * zrow + k) * ld + zb * zcol + n]);
    }
};

// Epilogue: C[m * ld + zb * zoff + n] = acc (+ bias[zb * zoff + n]), optionally also to a
// second buffer of another type.
template <typename T1, typename T2>
struct EpiRowMajor {
    T1 *c1; // nullable
    T2 *c2; // nullable
    i64 ld;
    const void *bias; // nullable, element type T1
    i64 zoff;
    __device__ __forceinline__ void operator()(int m, int n, float acc, int zb, int) const
    {
        const i64 col = zb * zoff + n;
        if (bias) acc += to_float(((const T1 *)bias)[col]);
        if (c1) c1[(i64)m * ld + col] = from_float<T1>(acc);
        if (c2) c2[(i64)m * ld + col] = from_float<T2>(acc);
    }
};

// Epilogue for float parameter gradients without k-split:
// C[(zb * zrow + m) * ld + zb * zcol + n] (+)= acc
struct EpiGrad {
    float *c;
    i64 ld;
    i64 zrow, zcol;
    int accumulate;
    __device__ __forceinline__ void operator()(int m, int n, float acc, int zb, int) const
    {
        float *dst = &c[(zb * zrow + m) * ld + zb * zcol + n];
        *dst = accumulate ? (*dst + acc) : acc;
    }
};

// Epilogue for k-split partial sums: P[ks][m * ld + zb * zoff + n] = acc  (count = M * ld per split)
struct EpiPartial {
    float *p;
    i64 ld, count;
    i64 zoff = 0;
    __device__ __forceinline__ void operator()(int m, int n, float acc, int zb, int ks) const
    {
        p[(i64)ks * count + (i64)m * ld + zb * zoff + n] = acc;
    }
};

int launch_splitk_reduce(hipStream_t stream, const float *partial, float *out, i64 count, int ksplit, int accumulate);
int launch_zero_f32(hipStream_t stream, float *out, i64 count);
// out[cols] (+)= column sums of src[rows x cols] (row stride ld); partial needs
// colsum_chunks(rows) * cols floats.
int colsum_chunks(i64 rows);
template <typename T>
int launch_colsum(hipStream_t stream, const T *src, float *partial, float *out, i64 rows, i64 cols, i64 ld,
                  int accumulate);

} // namespace pf
