// variants.hip.h -- table of tile variants and the launcher shared by the
// per-precision translation units.  Included once per precision with T fixed.
#pragma once
#include <atomic>

#include "gemm_kernel.hip.h"

namespace xg {

template <typename T> struct VariantEntry {
    const char *name;
    int mt_m, mt_n;
    int kt, wgm, wgn;   // slab depth, waves along m and n
    int wgs_per_cu;   // workgroups resident on one CU (register and LDS budget of the variant)
    float eff;        // fraction of the MFMA peak the variant sustains with its CU fully occupied (measured)
    float lone;       // what of that is left when a CU holds a single workgroup of the variant (measured)
    bool has_split;   // kernels with the split tail (GemmArgs::nsplit > 1) are built for this variant
    // launch(transA is K-contiguous, transB is K-contiguous, fast path allowed, args, stream)
    hipError_t (*launch)(bool ak, bool bk, bool fast, const GemmArgs<T> &g, hipStream_t st);
};

template <typename T, typename Cfg, bool AK, bool BK, bool FAST, bool SPLIT = false>
static hipError_t launch_one(const GemmArgs<T> &g, hipStream_t st) {
    auto kern = gemm_kernel<T, Cfg, AK, BK, FAST, SPLIT>;
    // LDS beyond 64 KiB has to be requested explicitly: once per kernel and device.
    if constexpr (Cfg::LDS_BYTES > 65536) {
        constexpr int MAX_DEV = 64;
        static std::atomic<int> done[MAX_DEV];          // 0: not yet, 1: granted
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
        if (done[dev].load(std::memory_order_acquire) == 0) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::LDS_BYTES);
            if (e != hipSuccess) return e;
            done[dev].store(1, std::memory_order_release);
        }
    }
    int64_t nt = tile_count(g.uplo, g.ntm, g.ntn, Cfg::MT_M, Cfg::MT_N);
    if (!SPLIT && g.kcut != 0) nt = (nt + 64 * NUM_XCD - 1) / (64 * NUM_XCD) * (64 * NUM_XCD);   // whole rounds of squares
    else if (!SPLIT && g.sub_count > 0) nt = 4 * (int64_t)g.sub_count;          // quarter tiles of the tail
    else if (!SPLIT && g.first > 0 && g.first < nt) nt = g.first;          // the leading tiles only
    if constexpr (SPLIT) {
        if (g.ndp < 0 || g.ndp > nt || g.nsplit < 1 || !g.part || !g.cnt) return hipErrorInvalidValue;
        nt = g.ndp + (nt - g.ndp) * g.nsplit;
    }
    if (nt > 0x7fffffff) return hipErrorInvalidValue;   // beyond one grid dimension (and any device memory)
    const dim3 grid((unsigned)nt), block(Cfg::NT);
    hipLaunchKernelGGL(kern, grid, block, Cfg::LDS_BYTES, st, g);
    return hipGetLastError();
}

// The element-wise fallback (FAST == false: leading dimensions too large for
// 32-bit slab offsets) is only built for the 64x64 tile; the host routes such
// calls to that variant.
template <typename T, typename Cfg, bool WITH_SPLIT = false>
static hipError_t launch_cfg(bool ak, bool bk, bool fast, const GemmArgs<T> &g0, hipStream_t st) {
    GemmArgs<T> g = g0;
    g.ntm = (g.m + Cfg::MT_M - 1) / Cfg::MT_M;
    g.ntn = (g.n + Cfg::MT_N - 1) / Cfg::MT_N;
    constexpr bool HAS_FALLBACK = (Cfg::MT_M == 64 && Cfg::MT_N == 64);
    if (g.nsplit > 1) {
        if constexpr (WITH_SPLIT) {
            if (!fast) return hipErrorInvalidValue;
            switch ((ak ? 2 : 0) | (bk ? 1 : 0)) {
                case 0: return launch_one<T, Cfg, false, false, true, true>(g, st);
                case 1: return launch_one<T, Cfg, false, true, true, true>(g, st);
                case 2: return launch_one<T, Cfg, true, false, true, true>(g, st);
                default: return launch_one<T, Cfg, true, true, true, true>(g, st);
            }
        }
        return hipErrorInvalidValue;
    }
    if (fast) {
        switch ((ak ? 2 : 0) | (bk ? 1 : 0)) {
            case 0: return launch_one<T, Cfg, false, false, true>(g, st);
            case 1: return launch_one<T, Cfg, false, true, true>(g, st);
            case 2: return launch_one<T, Cfg, true, false, true>(g, st);
            default: return launch_one<T, Cfg, true, true, true>(g, st);
        }
    }
    if constexpr (HAS_FALLBACK) {
        switch ((ak ? 2 : 0) | (bk ? 1 : 0)) {
            case 0: return launch_one<T, Cfg, false, false, false>(g, st);
            case 1: return launch_one<T, Cfg, false, true, false>(g, st);
            case 2: return launch_one<T, Cfg, true, false, false>(g, st);
            default: return launch_one<T, Cfg, true, true, false>(g, st);
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace xg
