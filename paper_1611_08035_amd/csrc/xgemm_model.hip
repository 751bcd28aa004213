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
//     pipe of its SIMD for 64 cycles (MFMA-only probe: 99 % of the published
//     peak = 1 MFMA / 64 cycles / SIMD);
//   * the LDS moves 128 bytes per cycle per CU, the vector-memory path takes
//     64 bytes per cycle per CU;
//   * the barrier of a slab (LDS writes drained, barrier, first fragment
//     reads) costs a SIMD about 180 cycles in which none of its waves issues
//     an MFMA (fitted to the KT = 16 and KT = 8 variants of the 128x128 tile).
constexpr double MFMA_CYCLES = 64.0;
constexpr double LDS_BYTES_PER_CLK = 128.0;
constexpr double VMEM_BYTES_PER_CLK = 64.0;
constexpr double BARRIER_STALL = 180.0;
constexpr int REG_BUDGET = 512;   // unified vector registers per SIMD lane

int vr(int tiles, int vec16) { return tiles % vec16 == 0 ? vec16 : (tiles % 2 == 0 ? 2 : 1); }
int ceil_div(int a, int b) { return (a + b - 1) / b; }
int shadow_quota(int n_mma, int n_ld, int n_rd, int n_wr) {
    for (int q = 1; q <= 4; ++q)
        if (ceil_div(n_ld, q) + ceil_div(n_rd, q) + ceil_div(n_wr, q) <= n_mma) return q;
    return 0;
}

template <typename T>
int predict(const xg::VariantEntry<T> &e, bool ak, bool bk, double *out) {
    const int es = (int)sizeof(T), vec16 = 16 / es;
    const int mi = es == 8 ? 16 : 32, ki = es == 8 ? 4 : 2, nr = es == 8 ? 4 : 16;
    const int nt = e.wgm * e.wgn * 64;
    const int tm = e.mt_m / e.wgm / mi, tn = e.mt_n / e.wgn / mi;
    const int ng = e.kt / ki, n_mma = tm * tn;
    const int nva = e.mt_m * e.kt / (nt * vec16), nvb = e.mt_n * e.kt / (nt * vec16);
    const int n_ld = nva + nvb;
    const int n_frag = tm / vr(tm, vec16) + tn / vr(tn, vec16);
    const int n_rd = ng * n_frag;
    const int n_wr = (ak ? nva * vec16 : nva) + (bk ? nvb * vec16 : nvb);
    const int waves_per_simd = e.wgs_per_cu * e.wgm * e.wgn / 4;
    const int waves_per_cu = waves_per_simd * 4;
    // pipelines, in cycles per slab
    const double t_mfma = (double)waves_per_simd * ng * n_mma * MFMA_CYCLES;                        // per SIMD
    const double rd_bytes = 64.0 * es * (tm + tn) * ng;                                             // per wave
    const double wr_bytes = 64.0 * 16.0 * n_ld;
    const double t_lds = waves_per_cu * (rd_bytes + wr_bytes) / LDS_BYTES_PER_CLK;                  // per CU
    const double t_vmem = waves_per_cu * (64.0 * 16.0 * n_ld) / VMEM_BYTES_PER_CLK;                 // per CU
    // outer-product rate = min over pipelines of rate / count (Sec. 4.2), with one
    // "job" per cycle of occupancy: rate 1, counts t_*
    const double rate[3] = {1.0, 1.0, 1.0};
    const double count[3] = {t_mfma, t_lds, t_vmem};
    const double slab_rate = xgemm_model_outer_product_rate(3, rate, count);
    // stall correction on the matrix pipe (Sec. 4.3): one barrier per slab
    const double w_mfma = t_mfma + 1.0 * BARRIER_STALL;
    const double slab_time = fmax(1.0 / slab_rate, w_mfma);
    const int q = shadow_quota((ng - 1) * n_mma, n_ld, (ng - 1) * n_frag, n_wr);
    const int regs = n_mma * nr * es / 4 + n_ld * 4 + 2 * (tm + tn) * es / 4;
    out[0] = ng * n_mma; out[1] = n_ld; out[2] = n_rd; out[3] = n_wr;
    out[4] = t_mfma; out[5] = t_lds; out[6] = t_vmem; out[7] = q;
    out[8] = BARRIER_STALL; out[9] = t_mfma / slab_time;
    out[10] = regs; out[11] = waves_per_simd;
    return (regs <= REG_BUDGET / waves_per_simd) ? 0 : 1;   // 1: the register limit of Sec. 5.4 is violated
}

}  // namespace

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

}  // extern "C"
