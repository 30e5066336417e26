// Host emulation of the stacked-LSTM entry points (test infrastructure, CPU only): the library's own host code is
// compiled with its launch macro redirected, so that every kernel launch becomes a CPU loop that does the kernel's
// arithmetic from its argument block and checks every operand range against a registry of the caller's buffers.
// What this exercises is the host logic - the diagonal schedule, the slice and workspace layout, the packed
// addressing that the copy kernels and their consumers must agree on - without a GPU.  Built by
// tests/test_host_lstm_stack.py; nothing in the product loads it.
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>
#include "pf_gemm.h"
#include "pf_skinny.h"

struct Buf { const char *p; size_t n; };
static std::vector<Buf> g_bufs;
static std::string g_err;
static int g_launches = 0;
extern "C" void emu_register(const void *p, size_t n) { g_bufs.push_back(Buf{(const char *)p, n}); }
extern "C" void emu_clear() { g_bufs.clear(); g_err.clear(); g_launches = 0; }
extern "C" const char *emu_error() { return g_err.c_str(); }
extern "C" int emu_launches() { return g_launches; }
static bool chk(const void *p, size_t count, const char *what)
{
    if (count == 0) return true;
    const char *c = (const char *)p;
    for (auto &b : g_bufs)
        if (c >= b.p && c + count * 4 <= b.p + b.n) return true;
    if (g_err.empty()) { char t[256]; snprintf(t, 256, "out of range: %s ptr %p count %zu", what, p, count); g_err = t; }
    return false;
}
#define CHK(p, n, w) do { if (!chk(p, n, w)) return PF_ERR_LAUNCH; } while (0)

namespace pf {
struct StackGatesFwd; struct StackGatesBwd; struct ZgPackArgs; struct ZgArgs; struct DgArgs;
template <int NRI> int emu_lstm_dhgates_kernel(dim3 grid, const DgArgs &a);
int emu_lstm_zg_pack_kernel(dim3 grid, const ZgPackArgs &a);
template <int NRI> int emu_lstm_zgates_kernel(dim3 grid, const ZgArgs &a);
int emu_lstm_stack_gates_fwd_kernel(dim3 grid, const StackGatesFwd &a);
int emu_lstm_stack_gates_bwd_kernel(dim3 grid, const StackGatesBwd &a);
template <int MODE> int emu_skinny_gemm_kernel(dim3 grid, const SkinnyArgs &a);
int emu_skinny_pack_kernel(dim3 grid, const SkinnyPackArgs &a);
int emu_slice_sum_kernel(dim3 grid, const SliceSumArgs &a);
int emu_rank_update_kernel(dim3 grid, const RankArgs &a, const SliceSumArgs &seg, int nsb);
template <int XI> int emu_rank_mma_kernel(dim3 grid, const RankMmaArgs &a);
int launch_zero_f32(hipStream_t, float *out, i64 count)
{
    if (count <= 0 || !out) return PF_OK;
    CHK(out, count, "zero");
    memset(out, 0, count * 4);
    return PF_OK;
}
}
#undef PF_LAUNCH
#define PF_LAUNCH(st, name, kernel, grid, block, s, ...) \
    do { if ((st) == PF_OK) { ++g_launches; (st) = emu_##kernel(grid, __VA_ARGS__); } } while (0)

#include "pf_skinny.hip"
#include "pf_rank_mma.hip"
#include "pf_lstm_stack.hip"

namespace pf {
int emu_skinny_pack_kernel(dim3 grid, const SkinnyPackArgs &a)
{
    if ((i64)grid.x * 256 < a.items) { g_err = "pack grid"; return PF_ERR_LAUNCH; }
    for (i64 g = 0; g < a.items; ++g) {
        int pi = 0;
        for (int q = 1; q < SK_MAX_PACK; ++q) if (q < a.n && g >= a.m[q].item0) pi = q;
        const SkinnyPackItem &m = a.m[pi];
        const i64 it = g - m.item0, S_total = (m.K + 7) / 8;
        const int lane = (int)(it & 63), e = (int)((it >> 6) & 3);
        const i64 S = (it >> 8) % S_total, tile = (it >> 8) / S_total;
        const i64 n = tile * SK_TILE_N + 32 * e + (lane & 31);
        CHK(m.dst + it * 4, 4, "pack dst");
        for (int s = 0; s < 4; ++s) {
            const i64 k = 8 * S + 4 * (lane >> 5) + s;
            float v = 0.f;
            if (k < m.K && n < m.N) { CHK(m.src + k * m.sk + n * m.sn, 1, "pack src"); v = m.src[k * m.sk + n * m.sn]; }
            m.dst[it * 4 + s] = v;
        }
    }
    return PF_OK;
}
template <int MODE> int emu_skinny_gemm_kernel(dim3 grid, const SkinnyArgs &a)
{
    constexpr bool NK = MODE == 1;
    int wg = 0;
    for (int q = 0; q < a.nprob; ++q) {
        const SkinnyProb &p = a.p[q];
        if (p.wg0 != wg) { g_err = "wg0 mismatch"; return PF_ERR_LAUNCH; }
        wg += p.ntiles * p.ksplit;
        for (int ks = 0; ks < p.ksplit; ++ks) {
            const int k0 = ks * p.kper, k1 = std::min(p.K, k0 + p.kper);
            for (int m = 0; m < p.M; ++m) {
                CHK(p.A + (i64)m * p.lda, p.K, "skinny A");
                CHK(p.P + (i64)ks * p.pcount + (i64)m * p.ldp, p.N, "skinny P");
                for (int n = 0; n < p.N; ++n) {
                    double acc = 0;
                    for (int k = k0; k < k1; ++k) {
                        const float *w = NK ? p.W + (i64)n * p.ldw + k : p.W + (i64)k * p.ldw + n;
                        if (MODE == 2) {
                            const i64 S_total = (p.K + 7) / 8;
                            const int lane = ((k % 8) / 4) * 32 + n % 32;
                            w = p.W + ((((i64)(n / 128) * S_total + k / 8) * 4 + (n % 128) / 32) * 64 + lane) * 4 + k % 4;
                            if (m == 0) CHK(w, 1, "skinny packed W");
                        } else
                        if (m == 0 && (NK ? k == k0 : n == 0)) CHK(w, NK ? (k1 - k0) : p.N, "skinny W");
                        acc += (double)p.A[(i64)m * p.lda + k] * *w;
                    }
                    p.P[(i64)ks * p.pcount + (i64)m * p.ldp + n] = (float)acc;
                }
            }
        }
    }
    if ((int)grid.x != wg) { g_err = "grid mismatch"; return PF_ERR_LAUNCH; }
    return PF_OK;
}
static int do_slice_sum(const SliceSumArgs &a)
{
    for (int q = 0; q < a.nseg; ++q) {
        const SliceSumSeg &s = a.s[q];
        for (int m = 0; m < s.M; ++m) {
            CHK(s.out + (i64)m * s.ldo, s.N, "slice out");
            if (s.bias) CHK(s.bias, s.N, "slice bias");
            for (int ks = 0; ks < s.ksplit; ++ks) CHK(s.P + (i64)ks * s.pcount + (i64)m * s.ldp, s.N, "slice P");
            for (int n = 0; n < s.N; ++n) {
                double acc = s.bias ? s.bias[n] : 0.0;
                for (int ks = 0; ks < s.ksplit; ++ks) acc += s.P[(i64)ks * s.pcount + (i64)m * s.ldp + n];
                s.out[(i64)m * s.ldo + n] = (float)acc;
            }
        }
    }
    return PF_OK;
}
int emu_slice_sum_kernel(dim3, const SliceSumArgs &a) { return do_slice_sum(a); }
int emu_rank_update_kernel(dim3 grid, const RankArgs &a, const SliceSumArgs &seg, int nsb)
{
    const int TI = 32; // rows of an output tile
    int tiles = 0;
    for (int q = 0; q < a.nprob; ++q) {
        const RankProb &p = a.p[q];
        if (p.wg0 != tiles) { g_err = "rank update: first workgroup of a problem"; return PF_ERR_LAUNCH; }
        tiles += ((p.I + TI - 1) / TI) * ((p.J + 127) / 128);
    }
    if (tiles != a.nwg || (int)grid.x != a.nwg + nsb) { g_err = "rank update: grid"; return PF_ERR_LAUNCH; }
    for (int q = 0; q < a.nprob; ++q) {
        const RankProb &p = a.p[q];
        for (int b = 0; b < p.M; ++b) {
            CHK(p.A + (i64)b * p.lda, p.I, "rank A");
            if (p.Bm) CHK(p.Bm + (i64)b * p.ldb, p.J, "rank B");
        }
        for (int i = 0; i < p.I; ++i) {
            CHK(p.out + (i64)i * p.ldo, p.J, "rank out");
            for (int j = 0; j < p.J; ++j) {
                double acc = a.accumulate ? p.out[(i64)i * p.ldo + j] : 0.0;
                for (int b = 0; b < p.M; ++b) acc += (double)p.A[(i64)b * p.lda + i] * (p.Bm ? p.Bm[(i64)b * p.ldb + j] : 1.0f);
                p.out[(i64)i * p.ldo + j] = (float)acc;
            }
        }
    }
    return nsb ? do_slice_sum(seg) : PF_OK;
}
template <int XI> int emu_rank_mma_kernel(dim3 grid, const RankMmaArgs &a)
{
    const int TI = 64 * XI;
    if (a.xi != XI) { g_err = "rank mma: tile height"; return PF_ERR_LAUNCH; }
    int tiles = 0;
    for (int q = 0; q < a.nprob; ++q) {
        const RankMmaProb &p = a.p[q];
        if (p.wg0 != tiles) { g_err = "rank mma: first workgroup of a problem"; return PF_ERR_LAUNCH; }
        if (p.M0 < 0 || p.M0 > p.M || p.M < 1) { g_err = "rank mma: rows"; return PF_ERR_LAUNCH; }
        if (p.I < 4 || p.J < 4) { g_err = "rank mma: a row shorter than four floats"; return PF_ERR_LAUNCH; }
        const int nt = ((p.I + TI - 1) / TI) * ((p.J + 127) / 128);
        if (p.ntile != nt || p.nwg != (nt + 7) / 8 * 8 || p.jt != (p.J + 127) / 128) { g_err = "rank mma: tiles of a problem"; return PF_ERR_LAUNCH; }
        tiles += p.nwg;
    }
    if (tiles != a.nwg || (int)grid.x != a.nwg) { g_err = "rank mma: grid"; return PF_ERR_LAUNCH; }
    for (int q = 0; q < a.nprob; ++q) {
        const RankMmaProb &p = a.p[q];
        auto row = [&](int b) { return b < p.M0 ? p.A0 + (i64)b * p.lda : p.A + (i64)(b - p.M0) * p.lda; };
        for (int b = 0; b < p.M; ++b) {
            CHK(row(b), p.I, "rank mma A");
            CHK(p.Bm + (i64)b * p.ldb, p.J, "rank mma B");
        }
        if (p.colsum) CHK(p.colsum, p.I, "rank mma column sums");
        for (int i = 0; i < p.I; ++i) {
            CHK(p.out + (i64)i * p.ldo, p.J, "rank mma out");
            for (int j = 0; j < p.J; ++j) {
                double acc = a.accumulate ? p.out[(i64)i * p.ldo + j] : 0.0;
                for (int b = 0; b < p.M; ++b) acc += (double)row(b)[i] * p.Bm[(i64)b * p.ldb + j];
                p.out[(i64)i * p.ldo + j] = (float)acc;
            }
            if (p.colsum) {
                double acc = a.accumulate ? p.colsum[i] : 0.0;
                for (int b = 0; b < p.M; ++b) acc += row(b)[i];
                p.colsum[i] = (float)acc;
            }
        }
    }
    return PF_OK;
}
static double sg(double z) { return 1.0 / (1.0 + exp(-z)); }
int emu_lstm_zg_pack_kernel(dim3 grid, const ZgPackArgs &a)
{
    const int S_total = (a.r + 7) / 8, E = a.mode == 0 ? 2 : 1;
    const int tiles = a.mode == 0 ? (a.h + ZG_HU - 1) / ZG_HU : (a.h + 31) / 32;
    const i64 per = (i64)tiles * S_total * 64 * E;
    if ((i64)grid.x * 256 < per * a.n) { g_err = "zg pack grid"; return PF_ERR_LAUNCH; }
    for (i64 g = 0; g < per * a.n; ++g) {
        const int mi = (int)(g / per);
        const i64 it = g % per;
        const int lane = (int)(it & 63), e = (int)((it >> 6) % E);
        const int S = (int)((it / (64 * E)) % S_total), tile = (int)((it / (64 * E)) / S_total);
        const int i = lane & 31;
        const int unit = a.mode == 0 ? tile * ZG_HU + (i & 15) : tile * 32 + i;
        const i64 row = a.mode == 0 ? (i64)(2 * e + (i >> 4)) * a.h + unit : unit;
        CHK(a.dst[mi] + it * 4, 4, "zg pack dst");
        for (int s4 = 0; s4 < 4; ++s4) {
            const int k = 8 * S + 4 * (lane >> 5) + s4;
            float v = 0.f;
            if (k < a.r && unit < a.h) { const float *src = a.src[mi] + row * a.r + k; CHK(src, 1, "zg pack src"); v = *src; }
            a.dst[mi][it * 4 + s4] = v;
        }
    }
    return PF_OK;
}
template <int NRI> int emu_lstm_dhgates_kernel(dim3 grid, const DgArgs &a)
{
    if (a.B > 4 * NRI) { g_err = "dg NRI"; return PF_ERR_LAUNCH; }
    const int B = a.B, h = a.h, r = a.r, r8 = (r + 7) & ~7, S_total = r8 / 8;
    int wg = 0;
    for (int li = 0; li < a.n; ++li) {
        const DgLayer &L = a.l[li];
        if (L.wg0 != wg) { g_err = "dg wg0"; return PF_ERR_LAUNCH; }
        wg += a.tiles;
        // the staging reads row-major [B x r] from A[0] (and A[1] with two pairs) whatever nseg is
        for (int seg = 0; seg < (L.nseg == 2 ? 2 : 1); ++seg) for (int row = 0; row < B; ++row) CHK(L.A[seg] + (i64)row * r, r, "dg A");
        for (int tile = 0; tile < a.tiles; ++tile) {
            // the first ring fill touches the tile's packed factors whatever nseg is
            CHK(L.W[0] + (i64)tile * S_total * 256, (size_t)S_total * 256, "dg W tile");
            for (int m = 0; m < B; ++m) for (int u = 0; u < 32; ++u) {
                const int unit = tile * 32 + u;
                if (unit >= h) continue;
                const i64 base = (i64)m * 4 * h + unit, idx = (i64)m * h + unit;
                double dh = 0;
                if (L.dh_a) { CHK(L.dh_a + idx, 1, "dg dh_a"); dh += L.dh_a[idx]; }
                if (L.dh_b) { CHK(L.dh_b + idx, 1, "dg dh_b"); dh += L.dh_b[idx]; }
                for (int seg = 0; seg < L.nseg; ++seg)
                    for (int k = 0; k < r; ++k) {
                        const int S = k / 8, lane = ((k % 8) / 4) * 32 + u;
                        const float *wp = L.W[seg] + (i64)tile * S_total * 256 + lane * 4 + (i64)S * 256 + k % 4;
                        if (m == 0) CHK(wp, 1, "dg W");
                        dh += (double)L.A[seg][(i64)m * r + k] * *wp;
                    }
                if (L.dh_out) { CHK(L.dh_out + idx, 1, "dg dh_out"); L.dh_out[idx] = dh; continue; }
                for (int g = 0; g < 4; ++g) { CHK(L.gates + base + (i64)g * h, 1, "dg gates"); CHK(L.dz + base + (i64)g * h, 1, "dg dz"); }
                CHK(L.c_prev + idx, 1, "dg c_prev"); CHK(L.c_out + idx, 1, "dg c_out"); CHK(L.dc_prev + idx, 1, "dg dc_prev");
                if (L.dc_next) CHK(L.dc_next + idx, 1, "dg dc_next");
                const double ig = L.gates[base], fg = L.gates[base + h], gg = L.gates[base + 2 * (i64)h], og = L.gates[base + 3 * (i64)h];
                const double tc = tanh(L.c_out[idx]);
                const double dc = (L.dc_next ? L.dc_next[idx] : 0.0) + dh * og * (1 - tc * tc);
                L.dc_prev[idx] = dc * fg;
                L.dz[base] = dc * gg * ig * (1 - ig);
                L.dz[base + h] = dc * L.c_prev[idx] * fg * (1 - fg);
                L.dz[base + 2 * (i64)h] = dc * ig * (1 - gg * gg);
                L.dz[base + 3 * (i64)h] = dh * tc * og * (1 - og);
            }
        }
    }
    if ((int)grid.x != wg) { g_err = "dg grid"; return PF_ERR_LAUNCH; }
    return PF_OK;
}
template <int NRI> int emu_lstm_zgates_kernel(dim3 grid, const ZgArgs &a)
{
    if (a.B > 4 * NRI) { g_err = "zg NRI"; return PF_ERR_LAUNCH; }
    const int B = a.B, h = a.h, r = a.r, r8 = (r + 7) & ~7, S_total = r8 / 8;
    int wg = 0;
    for (int li = 0; li < a.n; ++li) {
        const ZgLayer &L = a.l[li];
        if (L.wg0 != wg) { g_err = "zg wg0"; return PF_ERR_LAUNCH; }
        wg += a.tiles;
        for (int tile = 0; tile < a.tiles; ++tile) {
            for (int seg = 0; seg < L.nseg; ++seg) for (int row = 0; row < B; ++row) CHK(L.A[seg] + (i64)row * r, r, "zg A");
            for (int m = 0; m < B; ++m) for (int u = 0; u < ZG_HU; ++u) {
                const int unit = tile * ZG_HU + u;
                if (unit >= h) continue;
                double z[4];
                for (int g = 0; g < 4; ++g) {
                    const int e = g >> 1, i = (g & 1) * 16 + u;
                    double acc = 0;
                    for (int seg = 0; seg < L.nseg; ++seg)
                        for (int k = 0; k < r; ++k) {
                            const int S = k / 8, lane = ((k % 8) / 4) * 32 + i;
                            const float *wp = L.W[seg] + (i64)tile * S_total * 512 + lane * 4 + ((i64)S * 2 + e) * 256 + k % 4;
                            if (m == 0) CHK(wp, 1, "zg W");
                            acc += (double)L.A[seg][(i64)m * r + k] * *wp;
                        }
                    if (L.bias) { CHK(L.bias + (i64)g * h + unit, 1, "zg bias"); acc += L.bias[(i64)g * h + unit]; }
                    const i64 base = (i64)m * 4 * h + unit;
                    if (L.zadd) { CHK(L.zadd + base + (i64)g * h, 1, "zg zadd"); acc += L.zadd[base + (i64)g * h]; }
                    z[g] = acc;
                }
                const i64 base = (i64)m * 4 * h + unit, idx = (i64)m * h + unit;
                CHK(L.c_prev + idx, 1, "zg c_prev"); CHK(L.c_out + idx, 1, "zg c_out"); CHK(L.h_out + idx, 1, "zg h_out");
                for (int g = 0; g < 4; ++g) CHK(L.gates + base + (i64)g * h, 1, "zg gates");
                const double ig = sg(z[0]), fg = sg(z[1]), gg = tanh(z[2]), og = sg(z[3]);
                const double c = fg * L.c_prev[idx] + ig * gg;
                L.gates[base] = ig; L.gates[base + h] = fg; L.gates[base + 2 * (i64)h] = gg; L.gates[base + 3 * (i64)h] = og;
                L.c_out[idx] = c; L.h_out[idx] = og * tanh(c);
            }
        }
    }
    if ((int)grid.x != wg) { g_err = "zg grid"; return PF_ERR_LAUNCH; }
    return PF_OK;
}
int emu_lstm_stack_gates_fwd_kernel(dim3 grid, const StackGatesFwd &a)
{
    if ((int)grid.y != a.n || a.n < 1 || a.n > ST_MAX_LAYERS) { g_err = "gates grid"; return PF_ERR_LAUNCH; }
    if ((i64)grid.x * 256 < (i64)a.B * a.h) { g_err = "gates grid x"; return PF_ERR_LAUNCH; }
    const i64 Bh = (i64)a.B * a.h, pc = 4 * Bh;
    for (int q = 0; q < a.n; ++q) {
        CHK(a.P[q], (size_t)a.nslices[q] * pc, "gates P");
        if (a.bias[q]) CHK(a.bias[q], 4 * a.h, "gates bias");
        if (a.zadd[q]) CHK(a.zadd[q], pc, "gates zadd");
        CHK(a.c_prev[q], Bh, "gates c_prev"); CHK(a.h_out[q], Bh, "gates h_out"); CHK(a.c_out[q], Bh, "gates c_out");
        CHK(a.gates[q], pc, "gates gates");
        for (int b = 0; b < a.B; ++b) for (int j = 0; j < a.h; ++j) {
            double z[4];
            for (int g = 0; g < 4; ++g) {
                const i64 e = (i64)b * 4 * a.h + (i64)g * a.h + j;
                z[g] = 0;
                for (int s = 0; s < a.nslices[q]; ++s) z[g] += a.P[q][(i64)s * pc + e];
                if (a.bias[q]) z[g] += a.bias[q][g * a.h + j];
                if (a.zadd[q]) z[g] += a.zadd[q][e];
            }
            const double ig = sg(z[0]), fg = sg(z[1]), gg = tanh(z[2]), og = sg(z[3]);
            const i64 idx = (i64)b * a.h + j, base = (i64)b * 4 * a.h + j;
            const double c = fg * a.c_prev[q][idx] + ig * gg;
            a.gates[q][base] = ig; a.gates[q][base + a.h] = fg; a.gates[q][base + 2 * a.h] = gg; a.gates[q][base + 3 * a.h] = og;
            a.c_out[q][idx] = c; a.h_out[q][idx] = og * tanh(c);
        }
    }
    return PF_OK;
}
int emu_lstm_stack_gates_bwd_kernel(dim3 grid, const StackGatesBwd &a)
{
    if ((int)grid.y != a.n || a.n < 1 || a.n > ST_MAX_LAYERS) { g_err = "gates grid"; return PF_ERR_LAUNCH; }
    const i64 Bh = (i64)a.B * a.h, pc = 4 * Bh;
    for (int q = 0; q < a.n; ++q) {
        CHK(a.gates[q], pc, "bg gates"); CHK(a.c_prev[q], Bh, "bg c_prev"); CHK(a.c_out[q], Bh, "bg c_out");
        if (a.dh_a[q]) CHK(a.dh_a[q], Bh, "bg dh_a");
        if (a.dh_b[q]) CHK(a.dh_b[q], Bh, "bg dh_b");
        if (a.n1[q]) CHK(a.P1[q], (size_t)a.n1[q] * Bh, "bg P1");
        if (a.n2[q]) CHK(a.P2[q], (size_t)a.n2[q] * Bh, "bg P2");
        if (a.dc_next[q]) CHK(a.dc_next[q], Bh, "bg dc_next");
        CHK(a.dz[q], pc, "bg dz"); CHK(a.dc_prev[q], Bh, "bg dc_prev");
        for (int b = 0; b < a.B; ++b) for (int j = 0; j < a.h; ++j) {
            const i64 idx = (i64)b * a.h + j, base = (i64)b * 4 * a.h + j;
            double dh = (a.dh_a[q] ? a.dh_a[q][idx] : 0.0) + (a.dh_b[q] ? a.dh_b[q][idx] : 0.0);
            for (int k = 0; k < a.n1[q]; ++k) dh += a.P1[q][(i64)k * Bh + idx];
            for (int k = 0; k < a.n2[q]; ++k) dh += a.P2[q][(i64)k * Bh + idx];
            const float *gt = a.gates[q];
            const double ig = gt[base], fg = gt[base + a.h], gg = gt[base + 2 * a.h], og = gt[base + 3 * a.h];
            const double tc = tanh(a.c_out[q][idx]);
            const double dc = (a.dc_next[q] ? a.dc_next[q][idx] : 0.0) + dh * og * (1 - tc * tc);
            a.dc_prev[q][idx] = dc * fg;
            a.dz[q][base] = dc * gg * ig * (1 - ig);
            a.dz[q][base + a.h] = dc * a.c_prev[q][idx] * fg * (1 - fg);
            a.dz[q][base + 2 * a.h] = dc * ig * (1 - gg * gg);
            a.dz[q][base + 3 * a.h] = dh * tc * og * (1 - og);
        }
    }
    return PF_OK;
}
}
