// xgemm_model.hip -- the paper's analytical kernel-selection model (Sec. 4,
// Sec. 5.4) as host code, and its instantiation for the CDNA4 tile variants.
//
// Paper: pipelines are queues, functional units servers.  An outer product
// that puts L_i instructions into pipeline i, which retires lambda_i per
// cycle, proceeds at min_i lambda_i / L_i (Sec. 4.2); a pipeline with n
// dependent instructions of latency k needs W = L + n k instead of L
// (Sec. 4.3); the registers left after the accumulators and the column of A
// bound the number of unit updates in flight (Sec. 5.4).
//
// Here the "outer product" is one K slab of one workgroup's macro-tile, the
// pipelines are the matrix pipe of a SIMD, the LDS pipe and the vector-memory
// pipe of a CU, and the stall term is the one barrier per slab.
#include "../../include/xgemm.h"
#include "../../include/xgemm_probe.h"
#include "../../include/xgemm_tuning.h"
#include "tables.h"

#include <math.h>

namespace {

// CDNA4 (MI355X) issue table, the counterpart of the paper's per-CPU tables
// of latencies and ports.  Measured on the device, not taken from a manual:
//   * one v_mfma_f64_16x16x4_f64 or v_mfma_f32_32x32x2_f32 holds the matrix
//     pipe of its SIMD for 64 cycles, one v_mfma_f32_16x16x4_f32 for 32
//     (MFMA-only probe: 99 % of the published peak = 1 MFMA / 64 cycles / SIMD);
//   * the LDS moves 128 bytes per cycle per CU, the vector-memory path takes
//     64 bytes per cycle per CU;
//   * every K slab of every workgroup on a CU costs the matrix pipes about 110
//     cycles in which none of its waves issues an MFMA (LDS writes drained,
//     barrier, first fragment reads): the n k of Sec. 4.3's W = L + n k with
//     n = workgroups per CU.  Fitted to the measured full-occupancy efficiencies
//     of nine variants (32x32 to 256x128, two to eight workgroups per CU: loss
//     per slab 213, 326, 455, 880 cycles for 2, 3, 4, 8 workgroups); a slab with
//     only two MFMA groups (KT = 8 in fp64) hides less of it (x 1.4); a barrier
//     over eight waves instead of four is taken to cost the square of the ratio
//     (one variant to fit it to, so no more than a guess that is not far off).
constexpr double LDS_BYTES_PER_CLK = 128.0;
constexpr double VMEM_BYTES_PER_CLK = 64.0;
constexpr double BARRIER_STALL = 110.0;
constexpr double SHORT_SLAB_FACTOR = 1.4;
constexpr int REG_BUDGET = 512;      // unified vector registers per SIMD lane
constexpr int REG_FIXED = 30;        // offsets, LDS addresses, pointers, scalars of the epilogue
constexpr int LDS_PER_CU = 160 * 1024;

int vr(int tiles, int vec16) { return tiles % vec16 == 0 ? vec16 : (tiles % 2 == 0 ? 2 : 1); }
int ceil_div(int a, int b) { return (a + b - 1) / b; }
int shadow_quota(int n_mma, int n_ld, int n_rd, int n_wr) {
    for (int q = 1; q <= 4; ++q)
        if (ceil_div(n_ld, q) + ceil_div(n_rd, q) + ceil_div(n_wr, q) <= n_mma) return q;
    return 0;
}

// One point of the design space: an MFMA shape, a wave tile, a layout of waves, a slab depth.
struct Design {
    int es;                 // bytes per element
    int mi, ki, nr, cyc;    // MFMA tile, depth, result registers per lane (in elements), matrix-pipe cycles
    int wt_m, wt_n, wgm, wgn, kt;
};
struct Estimate {
    int n_mma_slab, n_ld, n_rd, n_wr, quota, regs, lds_bytes, wgs_fit;
    double t_mfma, t_lds, t_vmem, stall, util;
};

// Counts per K slab and wave, register and LDS need, how many workgroups a CU can hold, and the predicted
// matrix-pipe utilisation with `wgs` workgroups per CU (<= 0: as many as fit).
Estimate estimate(const Design &d, bool ak, bool bk, int wgs) {
    Estimate e{};
    const int vec16 = 16 / d.es, waves = d.wgm * d.wgn, nt = waves * 64;
    const int mt_m = d.wt_m * d.wgm, mt_n = d.wt_n * d.wgn;
    const int tm = d.wt_m / d.mi, tn = d.wt_n / d.mi, ng = d.kt / d.ki, n_mma = tm * tn;
    const int nva = mt_m * d.kt / (nt * vec16), nvb = mt_n * d.kt / (nt * vec16);
    const int n_frag = tm / vr(tm, vec16) + tn / vr(tn, vec16);
    e.n_mma_slab = ng * n_mma;
    e.n_ld = nva + nvb;
    e.n_rd = ng * n_frag;
    e.n_wr = (ak ? nva * vec16 : nva) + (bk ? nvb * vec16 : nvb);
    e.quota = shadow_quota((ng - 1) * n_mma, e.n_ld, (ng - 1) * n_frag, e.n_wr);
    // registers (Sec. 5.4): accumulators + staging of one slab + two fragment sets + fixed
    e.regs = n_mma * d.nr * d.es / 4 + e.n_ld * 4 + 2 * (tm + tn) * d.es / 4 + REG_FIXED;
    e.lds_bytes = 2 * d.kt * (mt_m + mt_n + 2 * vec16) * d.es;
    const int by_regs = e.regs <= REG_BUDGET ? (REG_BUDGET / e.regs) * 4 / waves : 0;   // waves per SIMD x 4 SIMDs / waves per workgroup
    const int by_lds = LDS_PER_CU / e.lds_bytes;
    e.wgs_fit = by_regs < by_lds ? by_regs : by_lds;
    if (e.wgs_fit > 8) e.wgs_fit = 8;
    if (wgs <= 0) wgs = e.wgs_fit;
    if (wgs <= 0) { e.util = 0.0; return e; }
    const double waves_per_simd = wgs * waves / 4.0, waves_per_cu = wgs * waves;
    e.t_mfma = waves_per_simd * e.n_mma_slab * d.cyc;                                              // per SIMD and slab
    const double rd_bytes = 64.0 * d.es * (tm + tn) * ng, wr_bytes = 64.0 * 16.0 * e.n_ld;          // per wave
    e.t_lds = waves_per_cu * (rd_bytes + wr_bytes) / LDS_BYTES_PER_CLK;                            // per CU
    e.t_vmem = waves_per_cu * (64.0 * 16.0 * e.n_ld) / VMEM_BYTES_PER_CLK;                         // per CU
    // Sec. 4.3: n stalls of k cycles on the matrix pipe; n = workgroups per CU (one barrier each per slab)
    double k_stall = BARRIER_STALL * (ng <= 2 ? SHORT_SLAB_FACTOR : 1.0) * (waves / 4.0) * (waves / 4.0);
    if (waves < 4) k_stall = BARRIER_STALL * (ng <= 2 ? SHORT_SLAB_FACTOR : 1.0);
    e.stall = wgs * k_stall;
    // Sec. 4.2: the slowest pipeline sets the pace; the matrix pipe's own time is Sec. 4.3's W = L + n k
    const double w_mfma = e.t_mfma / xgemm_model_stalled_rate(e.t_mfma, wgs, k_stall);
    const double rate[3] = {1.0, 1.0, 1.0}, count[3] = {w_mfma, e.t_lds, e.t_vmem};
    e.util = e.t_mfma * xgemm_model_outer_product_rate(3, rate, count);
    return e;
}

template <typename T> Design design_of(const xg::VariantEntry<T> &v) {
    const int es = (int)sizeof(T);
    return Design{es, es == 8 ? 16 : 32, es == 8 ? 4 : 2, es == 8 ? 4 : 16, 64,
                  v.mt_m / v.wgm, v.mt_n / v.wgn, v.wgm, v.wgn, v.kt};
}

template <typename T>
int predict(const xg::VariantEntry<T> &v, bool ak, bool bk, double *out) {
    const Design d = design_of(v);
    const Estimate e = estimate(d, ak, bk, v.wgs_per_cu);
    const int waves_per_simd = v.wgs_per_cu * v.wgm * v.wgn / 4;
    out[0] = e.n_mma_slab; out[1] = e.n_ld; out[2] = e.n_rd; out[3] = e.n_wr;
    out[4] = e.t_mfma; out[5] = e.t_lds; out[6] = e.t_vmem; out[7] = e.quota;
    out[8] = e.stall; out[9] = e.util;
    out[10] = e.regs; out[11] = waves_per_simd;
    return (waves_per_simd > 0 && e.regs <= REG_BUDGET / (waves_per_simd > 0 ? waves_per_simd : 1)) ? 0 : 1;
}

}  // namespace

namespace xg {
// Efficiency the planner uses for a variant: the model's where it agrees with the measured one to within
// MODEL_TOLERANCE, the measured one otherwise.
constexpr double MODEL_TOLERANCE = 0.025;
double planner_eff(const VariantEntry<double> &v) {
    const double m = estimate(design_of(v), false, true, v.wgs_per_cu).util;
    return fabs(m - (double)v.eff) <= MODEL_TOLERANCE ? m : (double)v.eff;
}
double planner_eff(const VariantEntry<float> &v) {
    const double m = estimate(design_of(v), false, true, v.wgs_per_cu).util;
    return fabs(m - (double)v.eff) <= MODEL_TOLERANCE ? m : (double)v.eff;
}
}  // namespace xg

extern "C" {

double xgemm_model_outer_product_rate(int n_pipes, const double *rate, const double *count) {
    double best = INFINITY;
    for (int i = 0; i < n_pipes; ++i)
        if (count[i] > 0.0) best = fmin(best, rate[i] / count[i]);
    return best;
}

double xgemm_model_stalled_rate(double L, double n_dependent, double latency) {
    return L / (L + n_dependent * latency);
}

int xgemm_model_n_updates(int r_total, int m_r, int n_r, int v, int r_a, int r_r) {
    if (v <= 0 || r_r <= 0) return -1;
    if (r_a <= 0) r_a = (m_r + v - 1) / v;
    return (int)floor(((double)r_total - (double)m_r * n_r / v - r_a) / r_r);
}

int xgemm_model_predict(char prec, int variant, char transa, char transb, double out[12]) {
    if (!out) return -5;
    const bool ak = !(transa == 'N' || transa == 'n'), bk = (transb == 'N' || transb == 'n');
    int nv = 0;
    if (prec == 'd' || prec == 'D') {
        const xg::VariantEntry<double> *t = xg::d_variant_table(&nv);
        if (variant < 0 || variant >= nv) return -2;
        return predict<double>(t[variant], ak, bk, out);
    }
    if (prec == 's' || prec == 'S') {
        const xg::VariantEntry<float> *t = xg::s_variant_table(&nv);
        if (variant < 0 || variant >= nv) return -2;
        return predict<float>(t[variant], ak, bk, out);
    }
    return -1;
}

int xgemm_model_efficiency(char prec, int variant, double out[3]) {
    if (!out) return -5;
    int nv = 0;
    if (prec == 'd' || prec == 'D') {
        const xg::VariantEntry<double> *t = xg::d_variant_table(&nv);
        if (variant < 0 || variant >= nv) return -2;
        out[0] = t[variant].eff;
        out[1] = estimate(design_of(t[variant]), false, true, t[variant].wgs_per_cu).util;
        out[2] = xg::planner_eff(t[variant]);
        return 0;
    }
    if (prec == 's' || prec == 'S') {
        const xg::VariantEntry<float> *t = xg::s_variant_table(&nv);
        if (variant < 0 || variant >= nv) return -2;
        out[0] = t[variant].eff;
        out[1] = estimate(design_of(t[variant]), false, true, t[variant].wgs_per_cu).util;
        out[2] = xg::planner_eff(t[variant]);
        return 0;
    }
    return -1;
}

int xgemm_model_enumerate(char prec, int cap, double *rows) {
    const bool dbl = prec == 'd' || prec == 'D';
    if (!dbl && prec != 's' && prec != 'S') return -1;
    if (cap < 0) return -2;
    if (cap > 0 && !rows) return -3;
    struct Shape { int mi, ki, nr, cyc; };
    const Shape d_shapes[] = {{16, 4, 4, 64}};
    const Shape s_shapes[] = {{32, 2, 16, 64}, {16, 4, 4, 32}};
    const Shape *shapes = dbl ? d_shapes : s_shapes;
    const int n_shapes = dbl ? 1 : 2, es = dbl ? 8 : 4;
    const int layouts[][2] = {{1, 1}, {2, 1}, {1, 2}, {2, 2}, {4, 2}, {2, 4}};
    int count = 0;
    auto keep = [&](const double (&r)[12]) {      // insertion into rows[], best predicted utilisation first
        if (cap == 0) return;
        int pos = count < cap ? count : cap;
        while (pos > 0 && (rows[(pos - 1) * 12 + 9] < r[9] ||
                           (rows[(pos - 1) * 12 + 9] == r[9] && rows[(pos - 1) * 12 + 10] * rows[(pos - 1) * 12 + 11] < r[10] * r[11])))
            --pos;
        if (pos >= cap) return;
        const int last = (count < cap ? count : cap - 1);
        for (int i = last; i > pos; --i)
            for (int c = 0; c < 12; ++c) rows[i * 12 + c] = rows[(i - 1) * 12 + c];
        for (int c = 0; c < 12; ++c) rows[pos * 12 + c] = r[c];
    };
    for (int si = 0; si < n_shapes; ++si)
        for (int wt_m = shapes[si].mi; wt_m <= 128; wt_m *= 2)
            for (int wt_n = shapes[si].mi; wt_n <= 128; wt_n *= 2)
                for (const auto &lay : layouts)
                    for (int kt = 8; kt <= 32; kt *= 2) {
                        const Design d{es, shapes[si].mi, shapes[si].ki, shapes[si].nr, shapes[si].cyc, wt_m, wt_n, lay[0], lay[1], kt};
                        const int nt = lay[0] * lay[1] * 64, vec16 = 16 / es;
                        const int mt_m = wt_m * lay[0], mt_n = wt_n * lay[1];
                        // the staging deals whole 16-byte vectors of a slab to the threads, and a fragment pair needs an even number of groups
                        if ((mt_m * kt) % (nt * vec16) || (mt_n * kt) % (nt * vec16) || (kt / shapes[si].ki) % 2) continue;
                        const Estimate e = estimate(d, false, true, 0);
                        // Sec. 5.4: the accumulators, one slab in flight and two fragment sets must fit a lane's registers
                        // at the occupancy the estimate assumes, and a workgroup must fit the LDS
                        if (e.wgs_fit < 1) continue;
                        const double r[12] = {(double)shapes[si].mi, (double)wt_m, (double)wt_n, (double)lay[0], (double)lay[1],
                                              (double)kt, (double)e.regs, (double)e.lds_bytes, (double)e.wgs_fit, e.util,
                                              (double)mt_m, (double)mt_n};
                        keep(r);
                        ++count;
                    }
    return count;
}

}  // extern "C"
