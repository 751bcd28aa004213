// xgemm_api.hip -- the C ABI: argument checks, quick returns, variant choice,
// launches; the split-plane complex GEMM as four real GEMMs; probes.
#include "../../include/xgemm.h"
#include "../../include/xgemm_probe.h"
#include "../../include/xgemm_tuning.h"
#include "tables.h"

#include <atomic>
#include <stdlib.h>
#include <string.h>

// Scratch of xgemm_dgemm_static (arrival counters, then partial tiles): lives in the code object, so every
// device the library runs on holds its own copy at its own address from load to process exit.  Host code
// never uses this name as an address; it asks the runtime for the device's copy once (static_scratch()).
#define XG_STATIC_CNT_BYTES 8192
static __device__ __align__(256) unsigned char scratch[XGEMM_STATIC_SCRATCH_BYTES];

namespace {

using namespace xg;

thread_local const char *t_last_kernel = "";
thread_local int t_forced_variant = -1;
thread_local int t_forced_split = -1;   // -1: the model decides; 0: plain tail; 1: quartered tail; S >= 2: S pieces where feasible
thread_local int t_last_split = 1;
// tuning knob (environment XGEMM_REQUIRE_ALIGNED=1): send operands that are not
// 16-byte aligned to the element-wise fallback instead of the buffer-load path
const bool t_require_aligned = getenv("XGEMM_REQUIRE_ALIGNED") != nullptr;

inline bool is_n(char t) { return t == 'N' || t == 'n'; }
inline bool is_t(char t) { return t == 'T' || t == 't' || t == 'C' || t == 'c'; }
inline bool is_c(char t) { return t == 'C' || t == 'c'; }
inline int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }
constexpr int64_t DIM_MAX = 0x7fffffff;   // tile indices and extents are 32-bit inside the kernels

template <typename T> const VariantEntry<T> *table(int *n);
template <> const VariantEntry<double> *table<double>(int *n) { return d_variant_table(n); }
template <> const VariantEntry<float> *table<float>(int *n) { return s_variant_table(n); }

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Number of compute units of the current device (256 on MI355X), read once per device.
int num_cus() {
    constexpr int MAX_DEV = 64;
    static std::atomic<int> cached[MAX_DEV];          // 0: not read yet
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return 256;
    if ((cus = cached[dev].load(std::memory_order_relaxed)) > 0) return cus;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
    cached[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

// Engine clock of the current device in GHz as the runtime reports it (2.4 on MI355X), read once per device;
// 2.4 where there is no device to ask (the planner is also called on hosts without one).
double clock_ghz() {
    constexpr int MAX_DEV = 64;
    static std::atomic<int> cached[MAX_DEV];          // kHz; 0: not read yet
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return 2.4;
    if ((khz = cached[dev].load(std::memory_order_relaxed)) <= 0) {
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess || khz < 500000 || khz > 5000000) return 2.4;
        cached[dev].store(khz, std::memory_order_relaxed);
    }
    return khz * 1e-6;
}

// Workspace of the *_ws entry points: arrival counters, then partial tiles.
constexpr size_t WS_CNT_BYTES = 8192;                       // 2048 counters
constexpr size_t WS_PART_BYTES = size_t(64) << 20;          // 512 tiles of 128 KiB
static_assert(WS_CNT_BYTES == XG_STATIC_CNT_BYTES && XGEMM_STATIC_SCRATCH_BYTES > WS_CNT_BYTES &&
                  XGEMM_STATIC_SCRATCH_BYTES <= WS_CNT_BYTES + WS_PART_BYTES, "static scratch: counters, then partial tiles");
constexpr int SPLIT_MAX = 32;                               // pieces per tile
constexpr int SPLIT_MIN_SLABS = 4;                          // K slabs a piece must keep

// Constants of the cost model below, measured on MI355X (times in microseconds).
constexpr double T_ROUND0 = 10.0;        // ramp-up and flush of a workgroup that nothing else hides
constexpr double PART_EFF = 0.96;        // a CU holding more than one but fewer than it has room for
constexpr double T_FLUSH0 = 2.0;         // per round of workgroups: what of their ramp-up and flush the others do not hide,
constexpr double T_FLUSH_KIB = 0.13;     //   T_FLUSH0 + T_FLUSH_KIB * (KiB of the C tile) / (workgroups per CU)
constexpr double REDUCE_GBS = 80.0;      // rate at which one workgroup reads partial tiles back
constexpr double PART_TBS = 6.0;         // rate at which all partial tiles are written and read
constexpr double T_SPLIT0 = 2.0;         // arrival counting
constexpr double B_HALF_LINE = 0.86;     // see make_plan
constexpr double T_LAUNCH = 4.0;         // a second launch on the same stream
constexpr double DRAIN_FRAC = 0.25;      // ... which starts only when the first has drained: the workgroups of its last round end
constexpr double T_DRAIN_MAX = 60.0;     // spread over about this fraction of that round's time, up to this much (measured:
                                         // 56 us at depth 1024, no more than that at depth 8192)
constexpr int64_t QUARTER_MIN_K = 1024;  // shallower products gain nothing from a quartered tail (measured)

struct Plan {
    int v;          // tile variant
    int nsplit;     // pieces per split tile (1: nothing is split)
    int64_t ndp;    // tiles computed whole
    int vq;         // >= 0: the tiles past ndp run as quarter tiles of this variant in a second launch
};

// Pick a tile variant, and whether to split the last partial round along K, with
// a small analytical cost model in the spirit of the paper's model-driven kernel
// selection (Sec. 4).  A CU works through a tile of depth k in
//   t(k) = 2 * tile_area * k / (CU peak * eff)
// whether it holds one tile or shares its matrix pipes between several.  The
// tiles of a variant run in rounds of (CUs x workgroups per CU); a full round
// costs wgs * t(k); the last, partly filled round costs occ * t(k) with occ
// workgroups per CU (a lone workgroup has nobody to hide its stalls behind:
// the variant's `lone` factor; more than one but fewer than fit: PART_EFF).  Every launch pays one
// ramp-up (at its start) and one flush (at its end) that nothing hides, T_ROUND0
// together, whether its last round is full or not.  With a workspace the rem
// tiles of that round may instead be cut into S <= slots / rem pieces of depth
// k / S each; that adds the write and read of rem * S partial tiles and the
// serial read of S partial tiles by the workgroup that finishes each tile.
// Without a workspace the rem tiles may instead run as 4 rem quarter tiles of the variant with
// half the tile size in both directions, in a second launch: a quarter of the depth-k work per
// workgroup, at that variant's efficiency, plus the launch.
template <typename T>
Plan make_plan(int64_t m, int64_t n, int64_t k, int uplo, const VariantEntry<T> *tab, int nv, bool fast,
               size_t lwork, bool b_kcontig = false) {
    const int64_t cus = num_cus();
    const double cu_flops_per_us = (sizeof(T) == 8 ? 32.0 : 64.0) * 4.0 * clock_ghz() * 1e3;   // flop / us
    Plan best{0, 1, 0, -1};
    double best_cost = 0.0;
    const bool forced_v = t_forced_variant >= 0 && t_forced_variant < nv;
    const int v_lo = forced_v ? t_forced_variant : 0, v_hi = forced_v ? t_forced_variant + 1 : nv;
    for (int v = v_lo; v < v_hi; ++v) {
        const VariantEntry<T> &e = tab[v];
        const int64_t tiles = tile_count(uplo, (int)((m + e.mt_m - 1) / e.mt_m), (int)((n + e.mt_n - 1) / e.mt_n),
                                         e.mt_m, e.mt_n);
        const int64_t slots = cus * e.wgs_per_cu;
        const double area = (double)e.mt_m * (double)e.mt_n;
        const double tile_bytes = area * sizeof(T);
        const int64_t full = tiles / slots, rem = tiles % slots;
        double eff_v = planner_eff(e);
        // fp32, op(B) K-contiguous, 128x128 tile with slabs of depth 16: a slab takes half a cache line from each
        // of 128 rows of B, and whether the other half is still near when the next slab wants it depends on the
        // size and on where the matrix lies: measured 0.73-0.95 of the variant's rate with nothing in between
        // (4096, 4352, 4608, 5000 slow on one box, 4096 and 4608 on another; never below two full rounds of
        // tiles).  From two rounds on the planner takes the low figure;
        // the depth-32 tile, which takes whole lines, or the 256x128 tile then win where they should.
        if (sizeof(T) == 4 && b_kcontig && e.mt_m == 128 && e.mt_n == 128 && e.kt == 16 && full >= 2) eff_v *= B_HALF_LINE;
        auto t_tile = [&](double depth) { return 2.0 * area * depth / (cu_flops_per_us * eff_v); };
        // per round: the read-modify-write of the C tiles is only partly hidden by the other workgroups of the
        // CU, the less so the larger the tile, the fewer of them and the shorter their K loops (fitted to rank-k
        // updates: 10.5 us per round of 128x128 tiles at k = 256, 3.9 at k = 1024)
        const double t_flush = (T_FLUSH0 + T_FLUSH_KIB * (tile_bytes / 1024.0) / (double)e.wgs_per_cu) *
                               (k < 256 ? 1.0 : 256.0 / (double)k);
        // a workgroup alone on its CU has nobody to hide its barriers and memory round trips behind; how much that
        // costs depends on the variant (least for the large tiles, most for the tile of one matrix instruction per
        // wave, which also waits for each instruction before it issues the next) and is measured per variant
        const double lone_eff = e.lone;
        auto t_tail = [&](int64_t units, double depth) {
            const int64_t occ = (units + cus - 1) / cus;
            return t_flush + (double)occ * t_tile(depth) / (occ == 1 ? lone_eff : occ < e.wgs_per_cu ? PART_EFF : 1.0);
        };
        // every launch ramps up once and flushes once with nothing to hide behind, whether its last
        // round is a full one or not
        const double rounds = T_ROUND0 + (double)full * (e.wgs_per_cu * t_tile((double)k) + t_flush);
        Plan p{v, 1, tiles, -1};
        double cost = rounds + (rem > 0 ? t_tail(rem, (double)k) : 0.0);
        if (rem > 0 && full > 0 && fast && t_forced_split != 0 && (k >= QUARTER_MIN_K || t_forced_split == 1)) {
            for (int w = 0; w < nv; ++w) {
                if (tab[w].mt_m * 2 != e.mt_m || tab[w].mt_n * 2 != e.mt_n) continue;
                const double qarea = (double)tab[w].mt_m * (double)tab[w].mt_n;
                const int64_t occ = (4 * rem + cus - 1) / cus;
                const double tq = 2.0 * qarea * (double)k / (cu_flops_per_us * planner_eff(tab[w]));
                // The second launch starts as the first one drains: its quarter tiles take the CUs as the large tiles
                // leave them and run beside the stragglers, so they neither pay a ramp-up of their own nor run alone;
                // the tail costs the longer of the drain and the quarter tiles' own time at their full rate
                // (measured at 3072^3: 100 us in fp64, 54 us in fp32).
                const double drain = DRAIN_FRAC * e.wgs_per_cu * t_tile((double)k);
                const double own = (double)occ * tq;
                const double capped = drain < T_DRAIN_MAX ? drain : T_DRAIN_MAX;
                const double c = rounds + T_LAUNCH + (capped > own ? capped : own);
                if (c < cost || t_forced_split == 1) { cost = c; p.ndp = full * slots; p.vq = w; }
                break;
            }
        }
        if (rem > 0 && e.has_split && fast && lwork > WS_CNT_BYTES && t_forced_split != 0 &&
            rem <= (int64_t)(WS_CNT_BYTES / sizeof(unsigned))) {
            const int64_t nslab = (k + e.kt - 1) / e.kt;
            const int64_t by_ws = (int64_t)((lwork - WS_CNT_BYTES) / ((size_t)rem * (size_t)tile_bytes));
            int64_t smax = slots / rem;
            if (smax > nslab / SPLIT_MIN_SLABS) smax = nslab / SPLIT_MIN_SLABS;
            if (smax > SPLIT_MAX) smax = SPLIT_MAX;
            if (smax > by_ws) smax = by_ws;
            auto t_split = [&](int64_t S) {
                return rounds + t_tail(rem * S, (double)k / (double)S) + T_SPLIT0 +
                       (double)S * tile_bytes / (REDUCE_GBS * 1e3) +
                       2.0 * (double)(rem * S) * tile_bytes / (PART_TBS * 1e6);
            };
            if (t_forced_split > 1 && smax >= 2) {       // tuning: take the forced count if it is feasible
                const int64_t S = t_forced_split < smax ? t_forced_split : smax;
                p.nsplit = (int)S;
                p.ndp = full * slots;
                p.vq = -1;
                cost = t_split(S);
            } else if (t_forced_split < 0) {
                for (int64_t S = 2; S <= smax; ++S) {
                    const double c = t_split(S);
                    if (c < cost) { cost = c; p.nsplit = (int)S; p.ndp = full * slots; p.vq = -1; }
                }
            }
        }
        if (v == v_lo || cost < best_cost) { best = p; best_cost = cost; }
    }
    return best;
}

// Clears the arrival counters of a workspace (a kernel, not a memset, so that a
// caller may capture it in a graph).
__global__ void __launch_bounds__(256) zero_words_kernel(unsigned *p, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// Address of the current device's copy of `scratch`, asked of the runtime on the first call on that device
// and kept (each device has its own copy at its own address).
void *static_scratch(hipError_t *err) {
    constexpr int MAX_DEV = 64;
    static std::atomic<void *> ptrs[MAX_DEV];
    int dev = 0;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= MAX_DEV) { *err = hipErrorInvalidDevice; return nullptr; }
    void *p = ptrs[dev].load(std::memory_order_acquire);
    if (p) return p;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err == hipSuccess && !p) *err = hipErrorInvalidSymbol;
    if (*err != hipSuccess) return nullptr;
    ptrs[dev].store(p, std::memory_order_release);
    return p;
}

// uplo: 0 general, 1 lower, 2 upper (the caller has checked m == n for those).
// static_ws: the workspace is the library's static scratch (xgemm_dgemm_static); work and lwork are ignored.
template <typename T>
int gemm_impl(char ta, char tb, int64_t m, int64_t n, int64_t k, T alpha, const T *A, int64_t lda,
              const T *B, int64_t ldb, T beta, T *C, int64_t ldc, void *stream, int uplo = 0, void *work = nullptr,
              size_t lwork = 0, int kcut = 0, int kaxis = 0, int kblk = 0, bool static_ws = false,
              int64_t a_panel = 0, int64_t b_panel = 0) {
    // a_panel, b_panel != 0: A and B are packed operands (GemmArgs::a_panel) whose sizes the caller has checked;
    // then ta = N, tb = T, lda = ldb = PACK_W and k is a multiple of every slab depth
    t_last_kernel = "none";
    t_last_split = 1;
    if (!is_n(ta) && !is_t(ta)) return -1;
    if (!is_n(tb) && !is_t(tb)) return -2;
    if (m < 0 || m > DIM_MAX) return -3;
    if (n < 0 || n > DIM_MAX) return -4;
    if (k < 0 || k > DIM_MAX) return -5;
    const bool ab_read = (alpha != T(0)) && m > 0 && n > 0 && k > 0;
    const int64_t rows_a = is_n(ta) ? m : k, rows_b = is_n(tb) ? k : n;
    if (ab_read && !A) return -7;
    if (!a_panel && lda < max64(1, rows_a)) return -8;
    if (ab_read && !B) return -9;
    if (!b_panel && ldb < max64(1, rows_b)) return -10;
    if (m > 0 && n > 0 && !C) return -12;
    if (ldc < max64(1, m)) return -13;

    if (m == 0 || n == 0) return 0;
    if (!ab_read && beta == T(1)) return 0;
    hipStream_t st = static_cast<hipStream_t>(stream);

    if (!ab_read) {
        t_last_kernel = "scale";
        const dim3 grid((unsigned)((m + 255) / 256), (unsigned)(n < 1024 ? n : 1024));
        hipLaunchKernelGGL(scale_kernel<T>, grid, dim3(256), 0, st, C, ldc, (int)m, (int)n, beta, uplo);
        return (int)hipGetLastError();
    }

    int nv = 0;
    const VariantEntry<T> *tab = table<T>(&nv);
    GemmArgs<T> g;
    g.A = A; g.B = B; g.C = C;
    g.lda = lda; g.ldb = ldb; g.ldc = ldc;
    g.m = (int)m; g.n = (int)n; g.k = (int)k;
    g.alpha = alpha; g.beta = beta;
    g.ntm = g.ntn = 0;
    g.uplo = uplo;
    g.a_panel = a_panel;
    g.b_panel = b_panel;
    // The buffer-load path addresses one slab (at most 256 rows or columns of
    // the stored operand) with 31-bit byte offsets; beyond that the element-wise
    // fallback runs.  16-byte loads of 4- or 8-byte aligned data are legal for
    // buffer instructions, so alignment of the bases or strides is not required.
    const int64_t ld_max = (int64_t(1) << 31) / (257 * (int64_t)sizeof(T));
    bool fast = lda <= ld_max && ldb <= ld_max;
    if (t_require_aligned)
        fast = fast && aligned16(A) && aligned16(B) && (lda * sizeof(T)) % 16 == 0 && (ldb * sizeof(T)) % 16 == 0;
    if (static_ws) {
        // What the same call would use of a full-size workspace must fit the static array; then the plan
        // below, made for the array's size, is that same plan.
        const Plan full = make_plan<T>(m, n, k, uplo, tab, nv, fast, WS_CNT_BYTES + WS_PART_BYTES, is_n(tb) && !b_panel);
        if (full.nsplit > 1) {
            const VariantEntry<T> &e = tab[full.v];
            const int64_t tiles = tile_count(uplo, (int)((m + e.mt_m - 1) / e.mt_m), (int)((n + e.mt_n - 1) / e.mt_n),
                                             e.mt_m, e.mt_n);
            const size_t need = WS_CNT_BYTES + (size_t)(tiles - full.ndp) * (size_t)full.nsplit * (size_t)e.mt_m *
                                                   (size_t)e.mt_n * sizeof(T);
            if (need > (size_t)XGEMM_STATIC_SCRATCH_BYTES) return XGEMM_E_SCRATCH;
        }
        hipError_t e = hipSuccess;
        work = static_scratch(&e);
        if (!work) return (int)e;
        lwork = XGEMM_STATIC_SCRATCH_BYTES;
    }
    if (!work || (reinterpret_cast<uintptr_t>(work) & 15u)) lwork = 0;
    const Plan plan = make_plan<T>(m, n, k, uplo, tab, nv, fast, lwork, is_n(tb) && !b_panel);
    int v = plan.v;
    if (!fast)   // the element-wise fallback exists for the 64x64 tile only
        for (int i = 0; i < nv; ++i)
            if (tab[i].mt_m == 64 && tab[i].mt_n == 64) v = i;
    g.ndp = 0;
    g.nsplit = 1;
    g.part = nullptr;
    g.cnt = nullptr;
    g.first = 0;
    g.sub_count = g.sub_base = g.sub_ntm = g.sub_ntn = 0;
    g.kcut = kcut;
    g.kaxis = kaxis;
    g.kblk = kblk;
    g.reverse = (kcut == 1 && kaxis == 0) ? 1 : 0;
    if (fast && plan.nsplit > 1) {
        g.ndp = (int)plan.ndp;
        g.nsplit = plan.nsplit;
        g.cnt = static_cast<unsigned *>(work);
        g.part = reinterpret_cast<T *>(static_cast<unsigned char *>(work) + WS_CNT_BYTES);
        t_last_split = plan.nsplit;
        if (static_ws) {
            // the array keeps whatever the last call (or an aborted one) left: the counters start at zero
            constexpr int N = (int)(WS_CNT_BYTES / sizeof(unsigned));
            hipLaunchKernelGGL(zero_words_kernel, dim3(N / 256), dim3(256), 0, st, g.cnt, N);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return (int)e;
        }
    }
    t_last_kernel = tab[v].name;
    // op(A) is K-contiguous when A is transposed; op(B) is K-contiguous when B is not
    if (kcut != 0 && (!fast || plan.nsplit != 1 || kblk % tab[v].mt_m != 0 || kblk % tab[v].mt_n != 0)) return (int)hipErrorInvalidValue;
    if (fast && plan.nsplit == 1 && plan.vq >= 0 && v == plan.v && kcut == 0) {
        // the full rounds with this variant, then the tail as quarter tiles of the smaller one
        const int big_ntm = (int)((m + tab[v].mt_m - 1) / tab[v].mt_m), big_ntn = (int)((n + tab[v].mt_n - 1) / tab[v].mt_n);
        const int64_t tiles = tile_count(uplo, big_ntm, big_ntn, tab[v].mt_m, tab[v].mt_n);
        g.first = (int)plan.ndp;
        const hipError_t e1 = tab[v].launch(is_t(ta), is_n(tb), fast, g, st);
        if (e1 != hipSuccess) return (int)e1;
        g.first = 0;
        g.sub_count = (int)(tiles - plan.ndp);
        g.sub_base = (int)plan.ndp;
        g.sub_ntm = big_ntm;
        g.sub_ntn = big_ntn;
        return (int)tab[plan.vq].launch(is_t(ta), is_n(tb), fast, g, st);
    }
    return (int)tab[v].launch(is_t(ta), is_n(tb), fast, g, st);
}

// C := alpha op(A) op(B) + beta C with both operands packed by xgemm_*pack_a / xgemm_*pack_b: the kernels of the
// N, T form with the tile origins taken from the panel layout.  The packed depth is a multiple of 32 and zero
// beyond k, so the product runs over the padded depth and never meets a ragged slab.
template <typename T>
int gemm_packed_impl(int64_t m, int64_t n, int64_t k, T alpha, const T *Ap, const T *Bp, T beta, T *C, int64_t ldc,
                     void *stream) {
    if (m < 0 || m > DIM_MAX) return -1;
    if (n < 0 || n > DIM_MAX) return -2;
    if (k < 0 || k > DIM_MAX) return -3;
    const bool ab_read = alpha != T(0) && m > 0 && n > 0 && k > 0;
    if (ab_read && !Ap) return -5;
    if (ab_read && !Bp) return -6;
    if (m > 0 && n > 0 && !C) return -8;
    if (ldc < max64(1, m)) return -9;
    const int64_t kpad = (k + 31) / 32 * 32;
    if (kpad > DIM_MAX) return -3;
    return gemm_impl<T>('N', 'T', m, n, kpad, alpha, Ap, PACK_W, Bp, PACK_W, beta, C, ldc, stream, 0, nullptr, 0, 0, 0, 0,
                        false, (int64_t)PACK_W * kpad, (int64_t)PACK_W * kpad);
}

// C := alpha op(A) op(A)^T + beta C on one triangle: the GEMM kernel with B = A,
// the opposite transpose, and the triangle mask.
template <typename T>
int syrk_impl(char uplo, char trans, int64_t n, int64_t k, T alpha, const T *A, int64_t lda, T beta, T *C,
              int64_t ldc, void *stream, void *work = nullptr, size_t lwork = 0) {
    t_last_kernel = "none";
    const bool lower = (uplo == 'L' || uplo == 'l'), upper = (uplo == 'U' || uplo == 'u');
    if (!lower && !upper) return -1;
    if (!is_n(trans) && !is_t(trans)) return -2;
    if (n < 0 || n > DIM_MAX) return -3;
    if (k < 0 || k > DIM_MAX) return -4;
    const bool a_read = (alpha != T(0)) && n > 0 && k > 0;
    if (a_read && !A) return -6;
    if (lda < max64(1, is_n(trans) ? n : k)) return -7;
    if (n > 0 && !C) return -9;
    if (ldc < max64(1, n)) return -10;
    // op(A) op(A)^T: second operand is the same matrix with the opposite transpose
    const int rc = gemm_impl<T>(is_n(trans) ? 'N' : 'T', is_n(trans) ? 'T' : 'N', n, n, k, alpha, A, lda, A, lda, beta,
                                C, ldc, stream, lower ? 1 : 2, work, lwork);
    return rc;   // the argument checks above cover every error gemm_impl could report
}

// C := alpha op(A) op(B)^T + alpha op(B) op(A)^T + beta C on one triangle: two launches of the GEMM
// kernel in triangle mode, the second accumulating onto the first.
template <typename T>
int syr2k_impl(char uplo, char trans, int64_t n, int64_t k, T alpha, const T *A, int64_t lda, const T *B, int64_t ldb,
               T beta, T *C, int64_t ldc, void *stream) {
    t_last_kernel = "none";
    const bool lower = (uplo == 'L' || uplo == 'l'), upper = (uplo == 'U' || uplo == 'u');
    if (!lower && !upper) return -1;
    if (!is_n(trans) && !is_t(trans)) return -2;
    if (n < 0 || n > DIM_MAX) return -3;
    if (k < 0 || k > DIM_MAX) return -4;
    const bool ab_read = (alpha != T(0)) && n > 0 && k > 0;
    if (ab_read && !A) return -6;
    if (lda < max64(1, is_n(trans) ? n : k)) return -7;
    if (ab_read && !B) return -8;
    if (ldb < max64(1, is_n(trans) ? n : k)) return -9;
    if (n > 0 && !C) return -11;
    if (ldc < max64(1, n)) return -12;
    const char t1 = is_n(trans) ? 'N' : 'T', t2 = is_n(trans) ? 'T' : 'N';
    const int ul = lower ? 1 : 2;
    // without a product term this is the scaling (or nothing) that the first call does by itself
    const int rc = gemm_impl<T>(t1, t2, n, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream, ul);
    if (rc || !ab_read) return rc;
    return gemm_impl<T>(t1, t2, n, n, k, alpha, B, ldb, A, lda, T(1), C, ldc, stream, ul);
}

// Elementwise combine for the complex path with complex scalars:
//   Cr = ar Pr - ai Pi + br Cr - bi Ci,   Ci = ar Pi + ai Pr + br Ci + bi Cr
// have_p == 0: the product term is absent (alpha == 0 or k == 0), P is not read.
// beta == 0: C is not read.
__global__ void __launch_bounds__(256) zcombine_kernel(double *Cr, double *Ci, int64_t ldc, const double *Pr,
                                                      const double *Pi, int m, int n, double ar, double ai,
                                                      double br, double bi, int have_p) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= m) return;
    const bool use_c = (br != 0.0 || bi != 0.0);
    for (int j = blockIdx.y; j < n; j += gridDim.y) {
        double xr = 0.0, xi = 0.0;
        if (have_p) {
            const double pr = Pr[i + (int64_t)j * m], pi = Pi[i + (int64_t)j * m];
            xr = ar * pr - ai * pi;
            xi = ar * pi + ai * pr;
        }
        double *cr = Cr + i + (int64_t)j * ldc, *ci = Ci + i + (int64_t)j * ldc;
        if (use_c) {
            const double c0 = *cr, c1 = *ci;
            xr += br * c0 - bi * c1;
            xi += br * c1 + bi * c0;
        }
        *cr = xr;
        *ci = xi;
    }
}

// Register-resident MFMA loop, no memory traffic: NACC independent accumulator
// tiles per wave (128 registers) so that back-to-back issue never waits on a
// dependency.
template <typename T> __global__ void __launch_bounds__(256, 2) mfma_peak_kernel(T *sink, int iters) {
    using M = Mfma<T>;
    constexpr int NACC = 128 / (M::NR * (int)sizeof(T) / 4);
    typename M::acc_t acc[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int r = 0; r < M::NR; ++r) acc[a][r] = T(0);
    T x = T(threadIdx.x & 7) * T(0.125), y = T((threadIdx.x >> 3) & 7) * T(0.25);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < NACC; ++a) acc[a] = M::mma(x, y, acc[a]);
    }
    T s = T(0);
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int r = 0; r < M::NR; ++r) s += acc[a][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// D = R * Cc with R(i, 0) = i, Cc(0, j) = 1 gives D(i, j) = i; with R(i, 0) = 1,
// Cc(0, j) = j gives D(i, j) = j.  Only k = 0 carries data.
template <typename T> __global__ void __launch_bounds__(64) mfma_layout_kernel(int *out) {
    using M = Mfma<T>;
    const int lane = threadIdx.x;
    const bool k0 = (M::op_k(lane) == 0);
    const T idx = T(M::op_idx(lane));
    typename M::acc_t di, dj;
#pragma unroll
    for (int r = 0; r < M::NR; ++r) { di[r] = T(0); dj[r] = T(0); }
    di = M::mma(k0 ? idx : T(0), k0 ? T(1) : T(0), di);
    dj = M::mma(k0 ? T(1) : T(0), k0 ? idx : T(0), dj);
#pragma unroll
    for (int r = 0; r < M::NR; ++r) out[lane * M::NR + r] = 256 * (int)di[r] + (int)dj[r];
}

// Latencies of dependent instruction chains as one lone wave sees them (the device's
// counterpart of the per-instruction latency column of the paper's micro-architecture
// table, Sec. 4.3: the k of W = L + n k).  Each section runs `iters` rounds of a chain
// in which every instruction needs the result of the one before, bracketed by the
// 100 MHz real-time counter; out[i] receives the ticks of section i (10 ns each):
//   0: 8 double-precision fused multiply-adds          1: 8 single-precision ones
//   2: 8 double-precision reciprocal square roots (each fed through one add)
//   3: 4 LDS round trips (write, read what another lane wrote)
//   4: 4 double-precision 16x16x4 matrix instructions accumulating into one tile
//   5: 4 times matrix instruction -> vector instruction on its result -> matrix instruction
//   6: 8 times lane read into scalar registers -> vector instruction that uses them
//   7: 4 single-precision 32x32x2 matrix instructions accumulating into one tile
__global__ void __launch_bounds__(64) latency_probe_kernel(long long *out, double *sink, int iters, double seed) {
    __shared__ double buf[64];
    const int lane = threadIdx.x;
    double x = seed + lane * 1e-9;
    const double y = 1.0000001;
    long long t[9];
    int n = 0;
    auto mark = [&] { t[n++] = wall_clock64(); };
    mark();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) x = __builtin_fma(x, y, 1e-12);
    }
    mark();
    {
        float xf = (float)x;
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int u = 0; u < 8; ++u) xf = __builtin_fmaf(xf, 1.0000001f, 1e-12f);
        }
        x = xf;
    }
    mark();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) x = __builtin_amdgcn_rsq(x + 2.0);
    }
    mark();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            buf[lane] = x;
            __builtin_amdgcn_wave_barrier();
            x = buf[(lane + 1) & 63] + 1e-12;
            __builtin_amdgcn_wave_barrier();
        }
    }
    mark();
    acc_d4 acc = {x, x, x, x};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x, y, acc, 0, 0, 0);
    }
    mark();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x, y, acc, 0, 0, 0);
            x = acc[0] * 1e-30 + 1.0;
        }
    }
    mark();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int lo = __builtin_amdgcn_readlane(__double2loint(x), (i + u) & 63);
            const int hi = __builtin_amdgcn_readlane(__double2hiint(x), (i + u) & 63);
            x = __builtin_fma(x, 1e-30, __hiloint2double(hi, lo));
        }
    }
    mark();
    acc_f16 accf;
#pragma unroll
    for (int r = 0; r < 16; ++r) accf[r] = (float)x;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) accf = __builtin_amdgcn_mfma_f32_32x32x2f32((float)y, 1.0f, accf, 0, 0, 0);
    }
    mark();
    sink[lane] = x + acc[1] + accf[3];
    if (lane == 0)
        for (int i = 0; i < 8; ++i) out[i] = t[i + 1] - t[i];
}

// One record per wave: {HW_ID, XCC_ID, blockIdx.x, wave in block}.  The block
// asks for `lds_bytes` of LDS so that its CU residency matches a GEMM kernel's.
__global__ void __launch_bounds__(256, 2) hwid_kernel(unsigned *out) {
    extern __shared__ unsigned char lds_dummy[];
    if (threadIdx.x == 0) lds_dummy[0] = 0;
    if ((threadIdx.x & 63) == 0) {
        const unsigned hw = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));
        const unsigned xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (31 << 11));
        unsigned *o = out + 4 * ((size_t)blockIdx.x * 4 + (threadIdx.x >> 6));
        o[0] = hw; o[1] = xcc; o[2] = blockIdx.x; o[3] = threadIdx.x >> 6;
    }
    // stay resident long enough that a full set of workgroups is live together
    const long long t0 = __builtin_readcyclecounter();
    while (__builtin_readcyclecounter() - t0 < 200000) {}
}

}  // namespace

namespace xg {
int gemm_cut(char ta, char tb, int64_t m, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
             const double *B, int64_t ldb, double *C, int64_t ldc, void *stream, int kcut, int kaxis, int kblk) {
    return gemm_impl<double>(ta, tb, m, n, k, alpha, A, lda, B, ldb, 1.0, C, ldc, stream, 0, nullptr, 0, kcut, kaxis, kblk);
}
int gemm_cut(char ta, char tb, int64_t m, int64_t n, int64_t k, float alpha, const float *A, int64_t lda,
             const float *B, int64_t ldb, float *C, int64_t ldc, void *stream, int kcut, int kaxis, int kblk) {
    return gemm_impl<float>(ta, tb, m, n, k, alpha, A, lda, B, ldb, 1.0f, C, ldc, stream, 0, nullptr, 0, kcut, kaxis, kblk);
}
}  // namespace xg

extern "C" {

int xgemm_dgemm(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha, const double *A,
                int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc, void *stream) {
    return gemm_impl<double>(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream);
}

int xgemm_dgemm_packed(int64_t m, int64_t n, int64_t k, double alpha, const double *Ap, const double *Bp, double beta,
                       double *C, int64_t ldc, void *stream) {
    return gemm_packed_impl<double>(m, n, k, alpha, Ap, Bp, beta, C, ldc, stream);
}

int xgemm_sgemm_packed(int64_t m, int64_t n, int64_t k, float alpha, const float *Ap, const float *Bp, float beta,
                       float *C, int64_t ldc, void *stream) {
    return gemm_packed_impl<float>(m, n, k, alpha, Ap, Bp, beta, C, ldc, stream);
}

int xgemm_sgemm(char transa, char transb, int64_t m, int64_t n, int64_t k, float alpha, const float *A,
                int64_t lda, const float *B, int64_t ldb, float beta, float *C, int64_t ldc, void *stream) {
    return gemm_impl<float>(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream);
}

int xgemm_dsyr2k(char uplo, char trans, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                 const double *B, int64_t ldb, double beta, double *C, int64_t ldc, void *stream) {
    return syr2k_impl<double>(uplo, trans, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream);
}

int xgemm_ssyr2k(char uplo, char trans, int64_t n, int64_t k, float alpha, const float *A, int64_t lda,
                 const float *B, int64_t ldb, float beta, float *C, int64_t ldc, void *stream) {
    return syr2k_impl<float>(uplo, trans, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream);
}

size_t xgemm_workspace_bytes(void) { return WS_CNT_BYTES + WS_PART_BYTES; }

int xgemm_workspace_init(void *work, size_t lwork, void *stream) {
    if (!work || (reinterpret_cast<uintptr_t>(work) & 15u)) return -1;
    if (lwork < WS_CNT_BYTES) return -2;
    constexpr int N = (int)(WS_CNT_BYTES / sizeof(unsigned));
    hipLaunchKernelGGL(zero_words_kernel, dim3(N / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<unsigned *>(work), N);
    return (int)hipGetLastError();
}

int xgemm_dgemm_ws(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha, const double *A,
                   int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc, void *work,
                   size_t lwork, void *stream) {
    if (work && (reinterpret_cast<uintptr_t>(work) & 15u)) return -14;
    return gemm_impl<double>(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream, 0, work, lwork);
}

int xgemm_dgemm_static(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha, const double *A,
                       int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc, void *stream) {
    return gemm_impl<double>(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream, 0, nullptr, 0, 0, 0, 0,
                             true);
}

int xgemm_sgemm_ws(char transa, char transb, int64_t m, int64_t n, int64_t k, float alpha, const float *A,
                   int64_t lda, const float *B, int64_t ldb, float beta, float *C, int64_t ldc, void *work,
                   size_t lwork, void *stream) {
    if (work && (reinterpret_cast<uintptr_t>(work) & 15u)) return -14;
    return gemm_impl<float>(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream, 0, work, lwork);
}

int xgemm_dsyrk_ws(char uplo, char trans, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                   double beta, double *C, int64_t ldc, void *work, size_t lwork, void *stream) {
    if (work && (reinterpret_cast<uintptr_t>(work) & 15u)) return -11;
    return syrk_impl<double>(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, stream, work, lwork);
}

int xgemm_ssyrk_ws(char uplo, char trans, int64_t n, int64_t k, float alpha, const float *A, int64_t lda, float beta,
                   float *C, int64_t ldc, void *work, size_t lwork, void *stream) {
    if (work && (reinterpret_cast<uintptr_t>(work) & 15u)) return -11;
    return syrk_impl<float>(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, stream, work, lwork);
}

int xgemm_plan(char prec, int uplo, int64_t m, int64_t n, int64_t k, size_t lwork, int out[3]) {
    if (uplo < 0 || uplo > 2) return -2;
    if (m <= 0 || m > DIM_MAX) return -3;
    if (n <= 0 || n > DIM_MAX) return -4;
    if (k <= 0 || k > DIM_MAX) return -5;
    if (!out) return -7;
    int nv = 0;
    Plan p;
    if (prec == 'd' || prec == 'D') {
        const VariantEntry<double> *t = d_variant_table(&nv);
        p = make_plan<double>(m, n, k, uplo, t, nv, true, lwork);
    } else if (prec == 's' || prec == 'S') {
        const VariantEntry<float> *t = s_variant_table(&nv);
        p = make_plan<float>(m, n, k, uplo, t, nv, true, lwork);
    } else {
        return -1;
    }
    out[0] = p.v;
    out[1] = p.nsplit;
    out[2] = (int)p.ndp;
    return 0;
}

void xgemm_tuning_reset(void) {
    t_forced_variant = -1;
    t_forced_split = -1;
    xg::reset_l3_tuning();
    xg::reset_lu_tuning();
}

int xgemm_force_split(int pieces) {
    if (pieces < -1 || pieces > SPLIT_MAX) return -1;
    t_forced_split = pieces;
    return 0;
}

int xgemm_last_split(void) { return t_last_split; }

int xgemm_dsyrk(char uplo, char trans, int64_t n, int64_t k, double alpha, const double *A, int64_t lda, double beta,
                double *C, int64_t ldc, void *stream) {
    return syrk_impl<double>(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, stream);
}

int xgemm_ssyrk(char uplo, char trans, int64_t n, int64_t k, float alpha, const float *A, int64_t lda, float beta,
                float *C, int64_t ldc, void *stream) {
    return syrk_impl<float>(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, stream);
}

int64_t xgemm_tile_map(int uplo, int64_t m, int64_t n, int mt_m, int mt_n, int *out, int64_t cap) {
    if (uplo < 0 || uplo > 2) return -1;
    if (m <= 0 || m > DIM_MAX) return -2;
    if (n <= 0 || n > DIM_MAX) return -3;
    if (mt_m <= 0) return -4;
    if (mt_n <= 0) return -5;
    const int ntm = (int)((m + mt_m - 1) / mt_m), ntn = (int)((n + mt_n - 1) / mt_n);
    const int64_t nt = tile_count(uplo, ntm, ntn, mt_m, mt_n);
    if (nt > DIM_MAX) return -2;
    if (out)
        for (int64_t b = 0; b < nt && b < cap; ++b) {
            const TilePos t = tile_of_lin(lin_of_block((int)b, (int)nt), ntm, ntn, uplo, mt_m, mt_n);
            out[2 * b] = t.tm;
            out[2 * b + 1] = t.tn;
        }
    return nt;
}

size_t xgemm_zgemm_worksize(int64_t m, int64_t n, const double alpha[2], const double beta[2]) {
    if (!alpha || !beta || m <= 0 || n <= 0) return 0;
    if (alpha[1] == 0.0 && beta[1] == 0.0) return 0;
    return (size_t)2 * (size_t)m * (size_t)n;
}

int xgemm_zgemm_split(char transa, char transb, int64_t m, int64_t n, int64_t k, const double alpha[2],
                      const double *Ar, const double *Ai, int64_t lda, const double *Br, const double *Bi,
                      int64_t ldb, const double beta[2], double *Cr, double *Ci, int64_t ldc, double *work,
                      int64_t lwork, void *stream) {
    t_last_kernel = "none";
    if (!is_n(transa) && !is_t(transa)) return -1;
    if (!is_n(transb) && !is_t(transb)) return -2;
    if (m < 0 || m > DIM_MAX) return -3;
    if (n < 0 || n > DIM_MAX) return -4;
    if (k < 0 || k > DIM_MAX) return -5;
    if (!alpha) return -6;
    if (!beta) return -13;
    const double ar = alpha[0], ai = alpha[1], br = beta[0], bi = beta[1];
    const bool ab_read = (ar != 0.0 || ai != 0.0) && m > 0 && n > 0 && k > 0;
    const int64_t rows_a = is_n(transa) ? m : k, rows_b = is_n(transb) ? k : n;
    if (ab_read && !Ar) return -7;
    if (ab_read && !Ai) return -8;
    if (lda < max64(1, rows_a)) return -9;
    if (ab_read && !Br) return -10;
    if (ab_read && !Bi) return -11;
    if (ldb < max64(1, rows_b)) return -12;
    if (m > 0 && n > 0 && !Cr) return -14;
    if (m > 0 && n > 0 && !Ci) return -15;
    if (ldc < max64(1, m)) return -16;
    const int64_t need = (int64_t)xgemm_zgemm_worksize(m, n, alpha, beta);
    if (need > 0 && !work) return -17;
    if (lwork < need) return -18;
    if (m == 0 || n == 0) return 0;
    if (!ab_read && br == 1.0 && bi == 0.0) return 0;

    // Im(op(X)) = sx * Xi : the conjugate only flips the sign of the imaginary plane.
    const double sa = is_c(transa) ? -1.0 : 1.0, sb = is_c(transb) ? -1.0 : 1.0;
    const char ta = is_n(transa) ? 'N' : 'T', tb = is_n(transb) ? 'N' : 'T';
    int rc;
    if (ai == 0.0 && bi == 0.0) {
        // real scalars: accumulate straight into the planes of C
        //   Cr = br Cr + ar Ar Br - ar sa sb Ai Bi ;  Ci = br Ci + ar sb Ar Bi + ar sa Ai Br
        if ((rc = xgemm_dgemm(ta, tb, m, n, k, ar, Ar, lda, Br, ldb, br, Cr, ldc, stream))) return rc;
        if ((rc = xgemm_dgemm(ta, tb, m, n, k, -ar * sa * sb, Ai, lda, Bi, ldb, 1.0, Cr, ldc, stream))) return rc;
        if ((rc = xgemm_dgemm(ta, tb, m, n, k, ar * sb, Ar, lda, Bi, ldb, br, Ci, ldc, stream))) return rc;
        if ((rc = xgemm_dgemm(ta, tb, m, n, k, ar * sa, Ai, lda, Br, ldb, 1.0, Ci, ldc, stream))) return rc;
        return 0;
    }
    // complex scalars: P = op(A) op(B) into the workspace, then one combine pass
    double *Pr = work, *Pi = work + (size_t)m * (size_t)n;
    if (ab_read) {
        if ((rc = xgemm_dgemm(ta, tb, m, n, k, 1.0, Ar, lda, Br, ldb, 0.0, Pr, m, stream))) return rc;
        if ((rc = xgemm_dgemm(ta, tb, m, n, k, -sa * sb, Ai, lda, Bi, ldb, 1.0, Pr, m, stream))) return rc;
        if ((rc = xgemm_dgemm(ta, tb, m, n, k, sb, Ar, lda, Bi, ldb, 0.0, Pi, m, stream))) return rc;
        if ((rc = xgemm_dgemm(ta, tb, m, n, k, sa, Ai, lda, Br, ldb, 1.0, Pi, m, stream))) return rc;
    }
    const dim3 grid((unsigned)((m + 255) / 256), (unsigned)(n < 1024 ? n : 1024));
    hipLaunchKernelGGL(zcombine_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), Cr, Ci, ldc, Pr, Pi,
                       (int)m, (int)n, ar, ai, br, bi, ab_read ? 1 : 0);
    return (int)hipGetLastError();
}

const char *xgemm_version(void) { return "xgemm 0.1 (gfx950)"; }

const char *xgemm_last_kernel_name(void) { return t_last_kernel; }

int xgemm_force_variant(int variant) {
    int nd = 0, ns = 0;
    d_variant_table(&nd);
    s_variant_table(&ns);
    if (variant < -1 || variant >= (nd > ns ? nd : ns)) return -1;
    t_forced_variant = variant;
    return 0;
}

const char *xgemm_variant_name(char prec, int variant) {
    int nv = 0;
    if (prec == 'd' || prec == 'D') {
        const VariantEntry<double> *t = d_variant_table(&nv);
        return (variant >= 0 && variant < nv) ? t[variant].name : nullptr;
    }
    if (prec == 's' || prec == 'S') {
        const VariantEntry<float> *t = s_variant_table(&nv);
        return (variant >= 0 && variant < nv) ? t[variant].name : nullptr;
    }
    return nullptr;
}

int xgemm_mfma_peak_probe(char prec, int blocks, int iters, void *sink, void *stream) {
    if (blocks <= 0 || iters < 0 || !sink) return (int)hipErrorInvalidValue;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (prec == 'd' || prec == 'D')
        hipLaunchKernelGGL(mfma_peak_kernel<double>, dim3(blocks), dim3(256), 0, st, static_cast<double *>(sink), iters);
    else if (prec == 's' || prec == 'S')
        hipLaunchKernelGGL(mfma_peak_kernel<float>, dim3(blocks), dim3(256), 0, st, static_cast<float *>(sink), iters);
    else
        return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

int xgemm_hwid_probe(int blocks, int lds_bytes, unsigned *out, void *stream) {
    if (blocks <= 0 || !out || lds_bytes < 0 || lds_bytes > 160 * 1024) return (int)hipErrorInvalidValue;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(hwid_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return (int)attr;
    hipLaunchKernelGGL(hwid_kernel, dim3(blocks), dim3(256), (size_t)lds_bytes, static_cast<hipStream_t>(stream), out);
    return (int)hipGetLastError();
}

int xgemm_latency_probe(long long *out, double *sink, int iters, void *stream) {
    if (!out || !sink || iters <= 0 || iters > (1 << 20)) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(latency_probe_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), out, sink, iters, 1.5);
    return (int)hipGetLastError();
}

int xgemm_mfma_layout_probe(char prec, int *out, void *stream) {
    if (!out) return (int)hipErrorInvalidValue;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (prec == 'd' || prec == 'D')
        hipLaunchKernelGGL(mfma_layout_kernel<double>, dim3(1), dim3(64), 0, st, out);
    else if (prec == 's' || prec == 'S')
        hipLaunchKernelGGL(mfma_layout_kernel<float>, dim3(1), dim3(64), 0, st, out);
    else
        return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

}  // extern "C"
