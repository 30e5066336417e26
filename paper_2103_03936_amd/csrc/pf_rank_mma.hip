// Weight gradients summed over hundreds of rows, on the matrix unit (fp32 32x32x2 MFMA).
//
// out[I][J] (+)= A^T * Bm with the summed index as the row of both operands in memory, which is exactly the order
// the MFMA wants: lane l of a k-pair supplies A[k = l / 32][i] and Bm[k = l / 32][j], so the chunks go into LDS as
// they lie in memory ([k][columns], no transposition, no padding) and every fragment read is conflict-free.
// A workgroup of four wavefronts owns a tile of 64 XI x 128 of out (XI = 1 or 2), a wavefront 32 XI x 64 of it in
// XI x 2 accumulators (independent MFMA chains); chunks of 32 rows are double-buffered in LDS, the global loads of
// the next two chunks in flight while a chunk is multiplied.  One workgroup per output tile and one accumulation
// order: deterministic.  The tile height is chosen per launch: whichever needs fewer rounds of workgroups over the
// chip, weighted by its height.  A bias gradient is the column sum of A: the first column tile of a problem adds it
// up from the chunks that pass through LDS anyway.
#include "pf_skinny.h"

namespace pf {

constexpr int RM_TJ = 128, RM_KC = 32; // tile width, rows per chunk

struct __attribute__((packed, aligned(4))) F2u {
    float v[2];
};
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

__device__ __forceinline__ const float *rank_mma_row(const RankMmaProb &pb, int b)
{
    return b < pb.M0 ? pb.A0 + (i64)b * pb.lda : pb.A + (i64)(b - pb.M0) * pb.lda;
}

// v[idx], idx in 0 .. 3, by selects (an index in a register would turn into branches)
__device__ __forceinline__ float pick4(f32x4_t v, int idx)
{
    float r = v[0];
    r = idx == 1 ? v[1] : r;
    r = idx == 2 ? v[2] : r;
    r = idx == 3 ? v[3] : r;
    return r;
}

// One tile of out.  FA / FB: all of the tile's rows / columns exist.  Otherwise a thread whose four columns would
// run past the row loads the row's last four instead (every load stays one 16-byte request, issued without a
// branch) and picks its elements out of them when the chunk is stored; what lies past the row is stored as zero.
template <int XI, bool FA, bool FB>
__device__ __forceinline__ void rank_mma_tile(const RankMmaProb &pb, int accumulate, int i0, int j0,
                                              float (*As)[RM_KC][64 * XI], float (*Bs)[RM_KC][RM_TJ])
{
    constexpr int TI = 64 * XI, NQA = TI / 32, RSA = 1024 / TI; // A: loads per thread and chunk, rows per pass
    const int tid = threadIdx.x, lane = tid & 63;
    const int I = pb.I, J = pb.J, M = pb.M;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = 32 * XI * (wave >> 1), wj = 64 * (wave & 1);
    // staging: of A a thread covers rows tid / (TI / 4) + RSA q (q < NQA), columns 4 (tid % (TI / 4)) .. + 3;
    // of Bm rows tid / 32 + 8 q (q < 4), columns 4 (tid % 32) .. + 3
    const int sra = tid / (TI / 4), sca = i0 + 4 * (tid % (TI / 4));
    const int srb = tid >> 5, scb = j0 + 4 * (tid & 31);
    const int la = FA ? sca : min(sca, I - 4), lb = FB ? scb : min(scb, J - 4); // where the loads start
    const int sha = sca - la, shb = scb - lb;

    // Two register sets: while chunk c is multiplied out of LDS, chunk c + 1 is on its way into one set (requested
    // one iteration earlier) and chunk c + 2 is requested into the other.  A request is two chunk-times old when
    // its data is needed.  Requests are unconditional: rows past the end come from the last row and are zeroed
    // when the chunk is stored, so the loop has no branch and the counters of outstanding loads stay exact.
    f32x4_t ra[2][NQA], rb[2][4];
    auto fetch = [&](int c, f32x4_t(&xa)[NQA], f32x4_t(&xb)[4]) {
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const int b = c * RM_KC + sra + RSA * q;
            xa[q] = ld4(rank_mma_row(pb, b < M ? b : M - 1) + la);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int b = c * RM_KC + srb + 8 * q;
            xb[q] = ld4(pb.Bm + (i64)(b < M ? b : M - 1) * pb.ldb + lb);
        }
    };
    auto stage = [&](int c, f32x4_t(&xa)[NQA], f32x4_t(&xb)[4]) {
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const bool live = c * RM_KC + sra + RSA * q < M;
            f32x4_t v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = FA ? xa[q][e] : pick4(xa[q], sha + e);
                v[e] = live && (FA || sca + e < I) ? t : 0.f;
            }
            *(f32x4_t *)&As[c & 1][sra + RSA * q][sca - i0] = v;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool live = c * RM_KC + srb + 8 * q < M;
            f32x4_t v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = FB ? xb[q][e] : pick4(xb[q], shb + e);
                v[e] = live && (FB || scb + e < J) ? t : 0.f;
            }
            *(f32x4_t *)&Bs[c & 1][srb + 8 * q][scb - j0] = v;
        }
    };

    f32x16_t acc[XI][2];
#pragma unroll
    for (int x = 0; x < XI; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;

    // The wavefront's block is split among its accumulators by parity: accumulator (x, y) holds the rows
    // wi + XI m + x and the columns wj + 2 n + y.  A lane's values of a k-pair are then neighbours in LDS: one read
    // for A, one for Bm.
    const int kl = lane >> 5, cl = lane & 31;
    auto read_a = [&](int buf, int k, float(&av)[XI]) {
        if (XI == 2) {
            const f32x2_t t = *(const f32x2_t *)&As[buf][k][wi + 2 * cl];
            av[0] = t[0];
            av[XI - 1] = t[1];
        } else {
            av[0] = As[buf][k][wi + cl];
        }
    };
    auto multiply = [&](int buf) {
        // fragments are read one k-pair ahead of the MFMAs that use them
        float fa[XI];
        read_a(buf, kl, fa);
        f32x2_t fb = *(const f32x2_t *)&Bs[buf][kl][wj + 2 * cl];
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0); // the first pair's LDS reads
#pragma unroll
        for (int kk = 0; kk < RM_KC / 2; ++kk) {
            float av[XI];
#pragma unroll
            for (int x = 0; x < XI; ++x) av[x] = fa[x];
            const f32x2_t bv = fb;
            if (kk + 1 < RM_KC / 2) {
                read_a(buf, 2 * kk + 2 + kl, fa);
                fb = *(const f32x2_t *)&Bs[buf][2 * kk + 2 + kl][wj + 2 * cl];
            }
#pragma unroll
            for (int x = 0; x < XI; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y)
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[x], bv[y], acc[x][y], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);      // the next pair's LDS reads
            __builtin_amdgcn_sched_group_barrier(0x008, 2 * XI, 0); // this pair's MFMAs
        }
    };

    // Column sums of A (a bias gradient) ride along in the first column tile of a problem that asks for them: each
    // thread adds a column's share of every chunk out of LDS, 256 / TI threads per column, in a fixed order.
    const bool cs = pb.colsum && j0 == 0;
    constexpr int CSP = 256 / TI, CSR = RM_KC / CSP; // threads per column, rows per thread and chunk
    float csum = 0.f;
    auto colsum = [&](int buf) {
        if (cs) {
#pragma unroll
            for (int e = 0; e < CSR; ++e) csum += As[buf][(tid / TI) * CSR + e][tid % TI];
        }
    };

    // an even number of chunks (a chunk past the end is all zeros), so that the register sets alternate statically
    const int nchunk = (M + 2 * RM_KC - 1) / (2 * RM_KC) * 2;
    fetch(0, ra[0], rb[0]);
    fetch(1, ra[1], rb[1]);
    stage(0, ra[0], rb[0]);
    __syncthreads();
    for (int c = 0; c < nchunk; c += 2) {
        // LDS buffer c & 1 holds chunk c; the other buffer was last read before the previous barrier.
        // (the scheduling fences keep the three phases apart, so that the dealing of LDS reads and MFMAs inside
        // multiply() is not mixed with the loads before it and the stores after it)
        fetch(c + 2, ra[0], rb[0]);
        __builtin_amdgcn_sched_barrier(0);
        multiply(0);
        __builtin_amdgcn_sched_barrier(0);
        colsum(0);
        stage(c + 1, ra[1], rb[1]);
        __syncthreads();
        fetch(c + 3, ra[1], rb[1]);
        __builtin_amdgcn_sched_barrier(0);
        multiply(1);
        __builtin_amdgcn_sched_barrier(0);
        colsum(1);
        stage(c + 2, ra[0], rb[0]);
        __syncthreads();
    }

    // accumulator element v of lane l is entry (m, n) = (8 (v / 4) + 4 (l / 32) + v % 4, l % 32) of its 32 x 32 block;
    // a lane stores the two neighbouring columns wj + 2 n, wj + 2 n + 1 together
    const int jj = j0 + wj + 2 * cl;
#pragma unroll
    for (int x = 0; x < XI; ++x)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int ii = i0 + wi + XI * (8 * (v >> 2) + 4 * kl + (v & 3)) + x;
            if (!FA && ii >= I) continue;
            float *o = pb.out + (i64)ii * pb.ldo + jj;
            if (FB || jj + 1 < J) {
                F2u t = {{acc[x][0][v], acc[x][1][v]}};
                if (accumulate) {
                    const F2u old = *(const F2u *)o;
                    t.v[0] += old.v[0];
                    t.v[1] += old.v[1];
                }
                *(F2u *)o = t;
            } else if (jj < J) {
                *o = accumulate ? *o + acc[x][0][v] : acc[x][0][v];
            }
        }
    if (cs) {
        // (every wavefront is past the loop's last barrier: the chunks in LDS are no longer needed)
        float *red = &Bs[0][0][0];
        red[tid] = csum;
        __syncthreads();
        if (tid < TI && i0 + tid < I) {
            float t = red[tid];
#pragma unroll
            for (int e = 1; e < CSP; ++e) t += red[e * TI + tid];
            float *o = pb.colsum + i0 + tid;
            *o = accumulate ? *o + t : t;
        }
    }
}

template <int XI>
__global__ __launch_bounds__(256, XI == 1 ? 3 : 2) void rank_mma_kernel(RankMmaArgs a)
{
    constexpr int TI = 64 * XI;
    __shared__ __attribute__((aligned(16))) float As[2][RM_KC][TI];
    __shared__ __attribute__((aligned(16))) float Bs[2][RM_KC][RM_TJ];
    int pi = 0;
#pragma unroll
    for (int q = 1; q < RM_MAX_PROB; ++q)
        if (q < a.nprob && (int)blockIdx.x >= a.p[q].wg0) pi = q;
    const RankMmaProb &pb = a.p[pi];
    const int local = blockIdx.x - pb.wg0;
    const int I = pb.I;

    // Workgroups go to the eight dies in turn, each die with an L2 of its own; a problem's workgroup count is a
    // multiple of eight and starts at one, so local % 8 is the die.  Tiles are dealt so that a die gets a run of
    // consecutive tiles: the column tiles of one row block, which read the same columns of A, then share its L2.
    const int per = pb.nwg / 8, tile = (local & 7) * per + (local >> 3);
    if (tile >= pb.ntile) return;
    const int i0 = (tile / pb.jt) * TI, j0 = (tile % pb.jt) * RM_TJ;
    const bool fa = i0 + TI <= I, fb = j0 + RM_TJ <= pb.J;
    if (fa && fb)
        rank_mma_tile<XI, true, true>(pb, a.accumulate, i0, j0, As, Bs);
    else if (fa)
        rank_mma_tile<XI, true, false>(pb, a.accumulate, i0, j0, As, Bs);
    else if (fb)
        rank_mma_tile<XI, false, true>(pb, a.accumulate, i0, j0, As, Bs);
    else
        rank_mma_tile<XI, false, false>(pb, a.accumulate, i0, j0, As, Bs);
}

bool rank_mma_add(RankMmaArgs &a, const float *A0, int M0, const float *A, i64 lda, const float *Bm, i64 ldb,
                  float *out, i64 ldo, int I, int J, int M, float *colsum)
{
    if (!out) return !colsum; // column sums ride on a matrix problem
    // the kernel's loads are four floats wide and pulled back inside a row: a row has to hold four
    if (a.nprob >= RM_MAX_PROB || M <= 0 || I < 4 || J < 4 || M0 < 0 || M0 > M) return false;
    RankMmaProb &p = a.p[a.nprob++];
    p.A0 = A0;
    p.A = A;
    p.Bm = Bm;
    p.out = out;
    p.colsum = colsum;
    p.lda = lda;
    p.ldb = ldb;
    p.ldo = ldo;
    p.M0 = M0;
    p.M = M;
    p.I = I;
    p.J = J;
    return true;
}

// tiles and first workgroups for tile height 64 xi; returns the tiles
static int rank_mma_plan(RankMmaArgs &a, int xi)
{
    a.nwg = 0;
    a.xi = xi;
    int tiles = 0;
    for (int q = 0; q < a.nprob; ++q) {
        RankMmaProb &p = a.p[q];
        p.jt = (p.J + RM_TJ - 1) / RM_TJ;
        p.ntile = ((p.I + 64 * xi - 1) / (64 * xi)) * p.jt;
        p.nwg = (p.ntile + 7) / 8 * 8;
        p.wg0 = a.nwg;
        a.nwg += p.nwg;
        tiles += p.ntile;
    }
    return tiles;
}

int launch_rank_mma(hipStream_t s, const char *name, const RankMmaArgs &args)
{
    int st = PF_OK;
    if (args.nprob <= 0) return st;
    RankMmaArgs a = args;
    // rounds of workgroups over the 256 compute units, weighted by the tile height; the taller tile on a tie (it
    // moves less data per multiply-add)
    const int t2 = rank_mma_plan(a, 2), t1 = rank_mma_plan(a, 1);
    const int c2 = 2 * ((t2 + 255) / 256), c1 = (t1 + 255) / 256;
    if (c1 < c2) {
        PF_LAUNCH(st, name, rank_mma_kernel<1>, dim3(a.nwg), dim3(256), s, a);
    } else {
        rank_mma_plan(a, 2);
        PF_LAUNCH(st, name, rank_mma_kernel<2>, dim3(a.nwg), dim3(256), s, a);
    }
    return st;
}

} // namespace pf
