// Truncated-SVD factor initialisation (Algorithm 1: W ~ U V^T with U = Ut_r S_r^(1/2), V = Vt_r S_r^(1/2)):
// one-sided Jacobi (Hestenes) in double precision.
//
// The matrix with fewer columns is taken (A = W or W^T, rows >= cols) and stored column-major, so that a column is
// contiguous.  A sweep orthogonalises every pair of columns once; pairs that share no column commute, so the
// cols (cols - 1) / 2 pairs of a sweep are dealt into cols - 1 rounds of cols / 2 disjoint pairs (round-robin
// tournament) and a round is one launch with a workgroup per pair: three dot products over the two columns, the
// plane rotation that zeroes their inner product, applied to the columns of A and of the accumulated right
// vectors Q.  When no pair of a sweep needed a rotation the remaining launches return at once.  Then
// singular values = column norms, sorted by counting, and the r largest triplets are scaled and written out.
#include "pf_gemm.h"

namespace pf {

constexpr int SVD_MAX_SWEEPS = 24;
// A pair counts as orthogonal when |a_p . a_q| <= tol |a_p| |a_q|.  The inner product of two columns of `rows`
// doubles carries rounding noise of about rows * 2^-53 relative to |a_p| |a_q|, so a tighter threshold never stops
// the sweeps; rows * 2^-52 still leaves the fp32 factors exact to their last bit.
static double svd_tolerance(int rows)
{
    const double t = (double)rows * 2.220446049250313e-16;
    return t < 1e-15 ? 1e-15 : t;
}

__global__ __launch_bounds__(256) void svd_init_kernel(const float *W, double *At, double *Qt, int n, int nr, int nc,
                                                        int transposed)
{
    const i64 idx = (i64)blockIdx.x * 256 + threadIdx.x;
    if (idx < (i64)nc * nr) {
        const int j = (int)(idx / nr), i = (int)(idx % nr);
        At[idx] = (double)(transposed ? W[(i64)j * n + i] : W[(i64)i * n + j]);
    }
    if (idx < (i64)nc * nc) Qt[idx] = (idx / nc == idx % nc) ? 1.0 : 0.0;
}

__global__ __launch_bounds__(256) void svd_round_kernel(double *At, double *Qt, int nr, int nc, int npad, int round,
                                                         int sweep, unsigned *rot, double tol)
{
    if (sweep > 0 && rot[sweep - 1] == 0u) return; // the sweep before found every pair orthogonal
    const int k = blockIdx.x, m1 = npad - 1, tid = threadIdx.x;
    int p = k == 0 ? m1 : (round + k) % m1, q = k == 0 ? round % m1 : (round - k + m1) % m1;
    if (p >= nc || q >= nc) return; // the padding player sits this round out
    if (p > q) {
        const int t = p;
        p = q;
        q = t;
    }
    double *ap = At + (i64)p * nr, *aq = At + (i64)q * nr;
    double alpha = 0.0, beta = 0.0, gamma = 0.0;
    for (int i = tid; i < nr; i += 256) {
        const double va = ap[i], vb = aq[i];
        alpha += va * va;
        beta += vb * vb;
        gamma += va * vb;
    }
    __shared__ double red[3][256];
    __shared__ double cs[2];
    __shared__ int rotate;
    red[0][tid] = alpha;
    red[1][tid] = beta;
    red[2][tid] = gamma;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) { // fixed tree: the same sums every run
        if (tid < s) {
            red[0][tid] += red[0][tid + s];
            red[1][tid] += red[1][tid + s];
            red[2][tid] += red[2][tid + s];
        }
        __syncthreads();
    }
    if (tid == 0) {
        alpha = red[0][0];
        beta = red[1][0];
        gamma = red[2][0];
        int doit = !(fabs(gamma) <= tol * sqrt(alpha * beta) || gamma == 0.0);
        if (doit) {
            const double zeta = (beta - alpha) / (2.0 * gamma);
            const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
            const double c = 1.0 / sqrt(1.0 + t * t);
            cs[0] = c;
            cs[1] = c * t;
            atomicAdd(&rot[sweep], 1u);
        }
        rotate = doit;
    }
    __syncthreads();
    if (!rotate) return;
    const double c = cs[0], s = cs[1];
    for (int i = tid; i < nr; i += 256) {
        const double va = ap[i], vb = aq[i];
        ap[i] = c * va - s * vb;
        aq[i] = s * va + c * vb;
    }
    double *qp = Qt + (i64)p * nc, *qq = Qt + (i64)q * nc;
    for (int i = tid; i < nc; i += 256) {
        const double va = qp[i], vb = qq[i];
        qp[i] = c * va - s * vb;
        qq[i] = s * va + c * vb;
    }
}

__global__ __launch_bounds__(256) void svd_sigma_kernel(const double *At, double *sig, int nr)
{
    const double *a = At + (i64)blockIdx.x * nr;
    double acc = 0.0;
    for (int i = threadIdx.x; i < nr; i += 256) acc += a[i] * a[i];
    __shared__ double red[256];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) sig[blockIdx.x] = sqrt(red[0]);
}

// position of column j in descending order of singular value (ties: lower index first)
__global__ __launch_bounds__(256) void svd_rank_kernel(const double *sig, int *rank, int nc)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= nc) return;
    const double s = sig[j];
    int k = 0;
    for (int i = 0; i < nc; ++i) k += (sig[i] > s || (sig[i] == s && i < j)) ? 1 : 0;
    rank[j] = k;
}

// column j of A (= sigma_j x left vector) and of Q (right vector) -> column rank[j] of the balanced factors
__global__ __launch_bounds__(256) void svd_emit_kernel(const double *At, const double *Qt, const double *sig,
                                                        const int *rank, float *U, float *V, float *sigma_out, int nr,
                                                        int nc, int r, int transposed, const unsigned *rot, int *info)
{
    if (info && blockIdx.x == 0 && threadIdx.x == 0) {
        // sweeps that ran (the first one that rotated nothing ends them) and rotations of the last one
        int ran = SVD_MAX_SWEEPS;
        for (int sw = 0; sw < SVD_MAX_SWEEPS; ++sw)
            if (rot[sw] == 0u) {
                ran = sw + 1;
                break;
            }
        info[0] = nc > 1 ? ran : 0;
        info[1] = nc > 1 ? (int)rot[ran - 1] : 0;
    }
    const int j = blockIdx.x, k = rank[j];
    const double s = sig[j];
    if (threadIdx.x == 0 && sigma_out) sigma_out[k] = (float)s;
    if (k >= r) return;
    const double rs = sqrt(s), inv = s > 0.0 ? rs / s : 0.0;
    float *left = transposed ? V : U, *right = transposed ? U : V;
    const double *a = At + (i64)j * nr, *qv = Qt + (i64)j * nc;
    for (int i = threadIdx.x; i < nr; i += 256) left[(i64)i * r + k] = (float)(a[i] * inv);
    for (int i = threadIdx.x; i < nc; i += 256) right[(i64)i * r + k] = (float)(qv[i] * rs);
}

struct SvdPlan {
    int nr, nc, npad, transposed;
    size_t n_At, n_Qt, bytes;
};
static int plan_svd(const pf_svd_desc *d, SvdPlan *p)
{
    if (!d) return PF_ERR_NULL;
    if (d->m <= 0 || d->n <= 0 || d->r <= 0) return PF_ERR_SHAPE;
    const i64 mn = d->m < d->n ? d->m : d->n, mx = d->m < d->n ? d->n : d->m;
    if (d->r > mn) return PF_ERR_SHAPE;
    if (mn > 8192 || mx > (1 << 24) || mn * mx > (1LL << 31)) return PF_ERR_UNSUPPORTED;
    p->transposed = d->m < d->n;
    p->nr = (int)mx;
    p->nc = (int)mn;
    p->npad = (p->nc + 1) / 2 * 2;
    p->n_At = (size_t)mn * mx;
    p->n_Qt = (size_t)mn * mn;
    p->bytes = align_up(p->n_At * 8) + align_up(p->n_Qt * 8) + align_up((size_t)mn * 8) + align_up((size_t)mn * 4) +
               align_up(64 * 4);
    return PF_OK;
}

} // namespace pf

using namespace pf;

extern "C" {

size_t pf_svd_split_workspace_bytes(const pf_svd_desc *d)
{
    SvdPlan p;
    return plan_svd(d, &p) == PF_OK ? p.bytes : 0;
}

int pf_svd_split(const pf_svd_desc *d, const void *W, void *U, void *V, void *sigma, void *info, void *workspace,
                 size_t workspace_bytes, void *stream)
{
    SvdPlan p;
    int st = plan_svd(d, &p);
    if (st != PF_OK) return st;
    if (!W || !U || !V) return PF_ERR_NULL;
    if (any_misaligned({W, U, V, sigma, info}, 4)) return PF_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < p.bytes) return PF_ERR_WORKSPACE;
    if (pf::any_misaligned({workspace}, 256)) return PF_ERR_UNSUPPORTED; // NULL passes: the size check has caught it
    Workspace ws(workspace, workspace_bytes);
    hipStream_t s = (hipStream_t)stream;
    double *At = ws.take<double>(p.n_At), *Qt = ws.take<double>(p.n_Qt), *sig = ws.take<double>(p.nc);
    int *rank = ws.take<int>(p.nc);
    unsigned *rot = ws.take<unsigned>(64);
    st = launch_zero_f32(s, (float *)rot, 64);
    if (st != PF_OK) return st;
    const i64 cells = (i64)p.nc * p.nr;
    PF_LAUNCH(st, "svd_init", svd_init_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), s, (const float *)W, At,
              Qt, (int)d->n, p.nr, p.nc, p.transposed);
    if (p.nc > 1) {
        for (int sweep = 0; sweep < SVD_MAX_SWEEPS && st == PF_OK; ++sweep)
            for (int round = 0; round < p.npad - 1 && st == PF_OK; ++round)
                PF_LAUNCH(st, "svd_jacobi_round", svd_round_kernel, dim3(p.npad / 2), dim3(256), s, At, Qt, p.nr, p.nc,
                          p.npad, round, sweep, rot, svd_tolerance(p.nr));
    }
    PF_LAUNCH(st, "svd_sigma", svd_sigma_kernel, dim3(p.nc), dim3(256), s, (const double *)At, sig, p.nr);
    PF_LAUNCH(st, "svd_rank", svd_rank_kernel, dim3((p.nc + 255) / 256), dim3(256), s, (const double *)sig, rank, p.nc);
    PF_LAUNCH(st, "svd_emit", svd_emit_kernel, dim3(p.nc), dim3(256), s, (const double *)At, (const double *)Qt,
              (const double *)sig, (const int *)rank, (float *)U, (float *)V, (float *)sigma, p.nr, p.nc, (int)d->r,
              p.transposed, (const unsigned *)rot, (int *)info);
    return st;
}

} // extern "C"
