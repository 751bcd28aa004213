// gemm_kernel.hip.h -- the GEMM macro/micro-kernel for CDNA4 (gfx950).
//
// The structure is the Goto/BLIS loop nest of the paper's Fig. 1 re-derived for
// the GPU memory hierarchy:
//
//   paper (CPU)                          here (MI355X)
//   ---------------------------------    -----------------------------------------
//   loops over n_c, m_c blocks of C      one workgroup per MT_M x MT_N macro-tile
//   loop over k_c + packing of A, B      K loop over KT-deep slabs; each slab of
//     into contiguous micro-panels         op(A), op(B) is staged HBM/L2 -> LDS in
//     (A column-major, B row-major,        [k][m] / [k][n] order (the same two
//     Sec. 2.1)                            layouts as the packed micro-panels)
//   micro-kernel: m_r x n_r block of C   one wavefront owns a WT_M x WT_N block of
//     in registers, loop of rank-1         C in accumulator registers for the whole
//     updates C += a_p b_p^T               K loop
//   unit update m_v x n_u (Sec. 2.2)     one MFMA instruction: a 16x16 (fp64) or
//                                          32x32 (fp32) block of C, rank-4 / rank-2
//   register budget (Sec. 5.4, the       accumulators + two operand fragment sets +
//     N_updates equation), no spills       in-flight global loads <= 256 VGPRs so two
//                                          waves share a SIMD; zero scratch
//   software pipelining: ramp-up /       global loads of slab t+1 (t+2 for the small
//     steady state / flush (Sec. 1,        tiles, TileCfg::PF) are issued before the
//     Sec. 5.5)                            MFMAs of slab t and written to the other
//                                          LDS buffer after them; one barrier per slab
//   C += c_reg (Fig. "code skeleton")    epilogue C = alpha*acc + beta*C, predicated
//                                          on the ragged edges
//
// Accumulator layout need not be the memory layout (the lesson of the paper's
// shuffle kernels, Sec. 3.2): the MFMA is fed op(B) as its row operand and
// op(A) as its column operand, i.e. it computes a block of C^T, so that the 16
// (or 32) consecutive lanes that hold one accumulator row map to consecutive
// rows m of column-major C and the epilogue's loads and stores are contiguous.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xg {

typedef double acc_d4 __attribute__((ext_vector_type(4)));
typedef float acc_f16 __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------
// MFMA traits: operand and accumulator register layouts (wave64).
//   operand:  lane l supplies element (idx = op_idx(l), k = op_k(l)) of the
//             MI x KI row operand, and (k = op_k(l), idx = op_idx(l)) of the
//             KI x MI column operand.
//   result :  register r of lane l holds D(d_row(l, r), d_col(l)).
// ---------------------------------------------------------------------------
template <typename T> struct Mfma;

template <> struct Mfma<double> {
    static constexpr int MI = 16, KI = 4, NR = 4;
    using acc_t = acc_d4;
    static __device__ __forceinline__ acc_t mma(double row_op, double col_op, acc_t c) {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(row_op, col_op, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int op_idx(int lane) { return lane & 15; }
    static __device__ __forceinline__ int op_k(int lane) { return lane >> 4; }
    static __device__ __forceinline__ int d_row(int lane, int r) { return (lane >> 4) + 4 * r; }
    static __device__ __forceinline__ int d_col(int lane) { return lane & 15; }
};

template <> struct Mfma<float> {
    static constexpr int MI = 32, KI = 2, NR = 16;
    using acc_t = acc_f16;
    static __device__ __forceinline__ acc_t mma(float row_op, float col_op, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(row_op, col_op, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int op_idx(int lane) { return lane & 31; }
    static __device__ __forceinline__ int op_k(int lane) { return lane >> 5; }
    static __device__ __forceinline__ int d_row(int lane, int r) {
        return (r & 3) + 4 * (lane >> 5) + 8 * (r >> 2);
    }
    static __device__ __forceinline__ int d_col(int lane) { return lane & 31; }
};

// N consecutive elements as one access (N = 1, 2 or 4); alignment of the
// element type only is promised to the compiler.
template <typename T, int N> struct Pack {
    typedef T type __attribute__((ext_vector_type(N), aligned(sizeof(T))));
    static __device__ __forceinline__ void load(const T *p, T (&out)[N]) {
        const type v = *reinterpret_cast<const type *>(p);
#pragma unroll
        for (int t = 0; t < N; ++t) out[t] = v[t];
    }
    static __device__ __forceinline__ void store(T *p, const T (&in)[N]) {
        type v;
#pragma unroll
        for (int t = 0; t < N; ++t) v[t] = in[t];
        *reinterpret_cast<type *>(p) = v;
    }
};
template <typename T> struct Pack<T, 1> {
    static __device__ __forceinline__ void load(const T *p, T (&out)[1]) { out[0] = *p; }
    static __device__ __forceinline__ void store(T *p, const T (&in)[1]) { *p = in[0]; }
};

template <typename T> struct GemmArgs {
    const T *A, *B;
    T *C;
    int64_t lda, ldb, ldc;
    int m, n, k;
    T alpha, beta;
    int ntm, ntn;   // macro-tiles along m and n
    int uplo;       // 0: all of C; 1: only the lower triangle (i >= j) is computed and written; 2: only the upper
    // Split tail (kernels built with SPLIT only).  The first `ndp` tiles of the
    // tile order are computed whole, one workgroup each; every later tile is cut
    // along K into `nsplit` pieces, one workgroup each, which leave their partial
    // sums in `part` (piece s of split tile q at part[(q*nsplit + s) * MT_M*MT_N])
    // and count themselves in cnt[q]; the piece that arrives last adds the
    // partial sums in the order s = 0, 1, ... and writes C.  cnt[] is zero before
    // the launch and zero again after it.  nsplit <= 1: nothing is split.
    int ndp, nsplit;
    T *part;
    unsigned *cnt;
    // Quartered tail (no workspace needed): a first launch computes only the first `first` tiles of the
    // order (0: all of them); a second launch with the variant of half the tile size in both directions
    // computes the remaining `sub_count` tiles as four quarter tiles each (sub_count > 0: workgroup b takes
    // quarter b & 3 of tile sub_base + (b >> 2) of the order over sub_ntm x sub_ntn tiles of twice the size).
    int first;
    int sub_count, sub_base, sub_ntm, sub_ntn;
    // Depth range that depends on the tile (the two passes of a symmetric product over the strict
    // triangles of its matrix; used with beta == 1 only).  With d = kblk * floor(x0 / kblk), x0 the
    // tile's first row (kaxis 0) or column (kaxis 1), and kblk a multiple of the tile size:
    // kcut 1 sums over k in [0, d), kcut 2 over [d + kblk, k); 0: all of k.  `reverse` walks the
    // tile order backwards (deepest tiles first for kcut 1 along the rows).
    int kcut, kaxis, kblk, reverse;
    // Packed operands (0: plain).  A packed op(A) is stored in panels of PACK_W rows, each panel a
    // PACK_W x Kpad column-major block (element (i, p) at [(i / PACK_W) * a_panel + p * PACK_W + i % PACK_W],
    // a_panel = PACK_W * Kpad, zero beyond the matrix), so that every slab of every tile is one run of
    // memory whatever the transpose or leading dimension of the source was; the call then has
    // lda = PACK_W and an MN-contiguous A.  The same for op(B)^T with b_panel.
    int64_t a_panel, b_panel;
};
constexpr int PACK_W = 256;

// ---------------------------------------------------------------------------
// Staging of one MT x KT slab of an operand from global memory into LDS in
// [k][mn] order with row stride S (the GPU form of the paper's packing).
//   KCONTIG == false: element (mn, p) is at base[mn + p*ld]  (A with trans=N, B with trans=T)
//   KCONTIG == true : element (mn, p) is at base[p + mn*ld]  (A with trans=T, B with trans=N)
// `base` points at the slab origin (tile row/col mn0, depth p0).
// Each thread moves NV vectors of 16 bytes; they sit in registers between the
// load (issued before the MFMAs of the current slab) and the LDS write (after).
// ---------------------------------------------------------------------------
template <typename T, int MT, int KT, int S, int NT, bool KCONTIG> struct Stager {
    static constexpr int V = 16 / (int)sizeof(T);
    static constexpr int NV = (MT * KT) / (NT * V);
    static_assert((MT * KT) % (NT * V) == 0, "slab must divide evenly over the threads");
    static_assert(KT % V == 0 && MT % V == 0, "vector width must divide the slab");
    typedef T vec_t __attribute__((ext_vector_type(V)));

    // Position of vector q of thread tid inside the slab: first element (mn, p).
    // MN-contiguous: consecutive threads walk along mn (coalesced 16-byte loads,
    // contiguous 16-byte LDS writes).
    // K-contiguous: a thread's vector holds V consecutive k of one mn and is
    // written to LDS as V scalars in V different rows (the transposition).  The
    // LDS serves W = 128 B / sizeof(T) lanes per cycle; with the row stride
    // S = MT + PADK (PADK = 16 B / sizeof(T)) lane group g of W lanes is laid out
    // as A = W / (PADK*V) k-chunks x B = W / A rows mn, whose bank offsets
    // PADK*V*kc + mn cover 0..W-1 exactly once: conflict-free.  Each group of
    // KP/A consecutive lane groups still covers whole rows of the slab, so the
    // global loads use every byte of the lines they touch.
    static constexpr int W = 128 / (int)sizeof(T);
    static constexpr int KP = KT / V;
    static constexpr int LA = (W / (V * V) < KP) ? W / (V * V) : KP;   // PADK == V (16 bytes)
    static constexpr int LB = W / LA;
    static __device__ __forceinline__ void pos(int tid, int q, int &mn, int &p) {
        const int v = tid + q * NT;
        if (!KCONTIG) {
            mn = (v % (MT / V)) * V;
            p = v / (MT / V);
        } else {
            const int kc = (v % LA) + LA * ((v / W) % (KP / LA));
            p = kc * V;
            mn = ((v / LA) % LB) + LB * (v / (W * (KP / LA)));
        }
    }

    // Byte offset of every vector of this thread from the slab origin.  They do
    // not change from slab to slab, so the steady-state loads are "uniform base
    // pointer + per-lane 32-bit offset" and need no vector address arithmetic.
    static __device__ __forceinline__ void offsets(uint32_t (&off)[NV], int64_t ld, int tid) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            int mn, p;
            pos(tid, q, mn, p);
            off[q] = (uint32_t)((KCONTIG ? p + (int64_t)mn * ld : mn + (int64_t)p * ld) * (int64_t)sizeof(T));
        }
    }

    // Buffer loads take the (wave-uniform) slab origin as a scalar resource and
    // the per-lane offset as a 32-bit register, so no vector ALU work is spent
    // on addresses.  The resource covers 2 GiB from the slab origin; an offset
    // at or beyond that is out of range and the load returns zero.
    static constexpr uint32_t RANGE = 0x80000000u;
    static __device__ __forceinline__ __amdgpu_buffer_rsrc_t resource(const T *base) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(base), 0, (int)RANGE, 0x00020000);
    }

    // the whole slab is in bounds: one 16-byte load per vector
    static __device__ __forceinline__ void load_fast(vec_t (&r)[NV], const T *base, const uint32_t (&off)[NV]) {
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        const __amdgpu_buffer_rsrc_t rsrc = resource(base);
#pragma unroll
        for (int q = 0; q < NV; ++q)
            r[q] = __builtin_bit_cast(vec_t, (u32x4)__builtin_amdgcn_raw_buffer_load_b128(rsrc, off[q], 0, 0));
    }

    // Ragged slab (edge tile or K tail): one load per element, zero-filled
    // outside [0, mn_lim) x [0, k_lim) by sending the out-of-range lanes' offsets
    // past the end of the resource -- no branches, all loads in flight together.
    static __device__ __forceinline__ void load_edge(vec_t (&r)[NV], const T *base, const uint32_t (&off)[NV],
                                                     int tid, int mn_lim, int k_lim) {
        const __amdgpu_buffer_rsrc_t rsrc = resource(base);
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            int mn, p;
            pos(tid, q, mn, p);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const int mne = KCONTIG ? mn : mn + e;
                const int pe = KCONTIG ? p + e : p;
                const uint32_t o = (mne < mn_lim && pe < k_lim) ? off[q] + e * (uint32_t)sizeof(T) : RANGE;
                if constexpr (sizeof(T) == 8) {
                    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
                    r[q][e] = __builtin_bit_cast(T, (u32x2)__builtin_amdgcn_raw_buffer_load_b64(rsrc, o, 0, 0));
                } else {
                    r[q][e] = __builtin_bit_cast(T, (unsigned int)__builtin_amdgcn_raw_buffer_load_b32(rsrc, o, 0, 0));
                }
            }
        }
    }

    // Edge tile, once per tile: vectors that lie wholly at or beyond mn_lim are sent
    // out of range for good (they load zeros in every slab), so that full-depth
    // slabs of an edge tile take the same 16-byte loads as an interior tile.  A
    // vector that straddles the limit (MN-contiguous slabs with mn_lim not a
    // multiple of V) is still loaded whole: what it picks up beyond the limit
    // comes from the same stored column of the operand and only ever feeds rows
    // or columns of C that are never stored.
    static __device__ __forceinline__ void trim(uint32_t (&off)[NV], int tid, int mn_lim) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            int mn, p;
            pos(tid, q, mn, p);
            if (mn >= mn_lim) off[q] = RANGE;
        }
    }
    // whether some vector of an edge tile straddles the limit (the same for every thread)
    static __device__ __forceinline__ bool straddles(int mn_lim) {
        return !KCONTIG && mn_lim < MT && (mn_lim % V) != 0;
    }

    // fallback without buffer addressing (leading dimensions too large for 32-bit
    // offsets): element-wise, zero-filled outside [0, mn_lim) x [0, k_lim)
    static __device__ __forceinline__ void load_guarded(vec_t (&r)[NV], const T *base, int64_t ld, int tid,
                                                        int mn_lim, int k_lim) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            int mn, p;
            pos(tid, q, mn, p);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const int mne = KCONTIG ? mn : mn + e;
                const int pe = KCONTIG ? p + e : p;
                T x = T(0);
                if (mne < mn_lim && pe < k_lim)
                    x = KCONTIG ? base[pe + (int64_t)mne * ld] : base[mne + (int64_t)pe * ld];
                r[q][e] = x;
            }
        }
    }

    // LDS position of vector 0 of this thread; vector q sits a compile-time
    // constant further on (rows for MN-contiguous slabs, columns for K-contiguous).
    static_assert(NT % (KCONTIG ? W * (KP / LA) : MT / V) == 0, "vectors of one thread must differ by a constant");
    static_assert(!KCONTIG || (KP % LA == 0 && W / (V * V) <= KP), "K-contiguous lane layout needs KT >= W / V");
    static __device__ __forceinline__ int lds_origin(int tid) {
        int mn, p;
        pos(tid, 0, mn, p);
        return p * S + mn;
    }
    static constexpr int lds_step = KCONTIG ? NT / (KT / V) : (NT / (MT / V)) * S;

    // `s` already includes lds_origin(tid)
    static __device__ __forceinline__ void store(const vec_t (&r)[NV], T *s) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            if (!KCONTIG) {
                *reinterpret_cast<vec_t *>(s + q * lds_step) = r[q];
            } else {
#pragma unroll
                for (int e = 0; e < V; ++e) s[e * S + q * lds_step] = r[q][e];
            }
        }
    }
};

// COUNT instructions of class MASK dealt PER at a time behind one MFMA each: a
// hint asking the scheduler to issue every memory instruction in the shadow of
// an MFMA.  An MFMA occupies the matrix pipe for 64 cycles during which this
// wave could not issue another one anyway, so one or two LDS or global
// instructions placed there are free, whereas a cluster of them stalls the pipe.
template <int MASK, int COUNT, int PER = 1> static __device__ __forceinline__ void interleave() {
    if constexpr (COUNT > 0) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(MASK, COUNT < PER ? COUNT : PER, 0);
        interleave<MASK, (COUNT > PER ? COUNT - PER : 0), PER>();
    }
}
constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }
// smallest number of memory instructions per MFMA with which n_ld + n_rd + n_wr
// of them fit behind n_mma MFMAs (0 if even 4 per MFMA do not)
constexpr int shadow_quota(int n_mma, int n_ld, int n_rd, int n_wr) {
    for (int q = 1; q <= 4; ++q)
        if (ceil_div(n_ld, q) + ceil_div(n_rd, q) + ceil_div(n_wr, q) <= n_mma) return q;
    return 0;
}

// blockIdx -> macro-tile.  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2: give every XCD one contiguous run of the tile order, and
// walk that order in bands of GROUP_M tile-rows so that the tiles resident on
// an XCD at one time share A row-panels and B column-panels.
static constexpr int NUM_XCD = 8;
static constexpr int GROUP_M = 8;

// Triangular results (uplo 1: lower, 2: upper): inside a band of tile-rows
// [first, first + gsz) only the tiles that reach the triangle are in the order.
// The columns of the band fall into a run whose tiles are all needed ("whole"
// columns [w0, w1)) and a short run beside the diagonal with fewer rows each
// ("cut" columns [p0, p1), at most gsz * mt_m / mt_n + 1 of them); the cut run
// follows the whole run for the lower triangle and precedes it for the upper.
struct Band { int w0, w1, p0, p1; };
static __host__ __device__ __forceinline__ int min_i(int64_t a, int64_t b) { return (int)(a < b ? a : b); }
static __host__ __device__ __forceinline__ Band band_of(int uplo, int first, int gsz, int ntn, int mt_m, int mt_n) {
    Band b;
    if (uplo == 1) {
        // column tn is needed from row floor(tn*mt_n / mt_m) on
        b.w0 = 0;
        b.w1 = min_i(ntn, ((int64_t)(first + 1) * mt_m - 1) / mt_n + 1);
        b.p0 = b.w1;
        b.p1 = min_i(ntn, ((int64_t)(first + gsz) * mt_m - 1) / mt_n + 1);
    } else {
        // column tn is needed up to row floor(((tn+1)*mt_n - 1) / mt_m)
        b.p0 = min_i(ntn, ((int64_t)first * mt_m) / mt_n);
        b.p1 = min_i(ntn, ((int64_t)(first + gsz - 1) * mt_m) / mt_n);
        b.w0 = b.p1;
        b.w1 = ntn;
    }
    return b;
}
// rows [r0, r0 + cnt) of the band that column tn needs
struct ColRows { int r0, cnt; };
static __host__ __device__ __forceinline__ ColRows col_rows(int uplo, int first, int gsz, int tn, int mt_m, int mt_n) {
    if (uplo == 1) {
        const int lo = (int)(((int64_t)tn * mt_n) / mt_m);
        const int r0 = lo > first ? lo : first;
        return ColRows{r0, first + gsz - r0};
    }
    const int hi = (int)((((int64_t)tn + 1) * mt_n - 1) / mt_m) + 1;
    return ColRows{first, (hi < first + gsz ? hi : first + gsz) - first};
}
static __host__ __device__ __forceinline__ int band_size(int uplo, int first, int gsz, int ntn, int mt_m, int mt_n) {
    const Band b = band_of(uplo, first, gsz, ntn, mt_m, mt_n);
    int sz = gsz * (b.w1 - b.w0);
    for (int tn = b.p0; tn < b.p1; ++tn) sz += col_rows(uplo, first, gsz, tn, mt_m, mt_n).cnt;
    return sz;
}

// Number of workgroups to launch (without split tiles).
static __host__ __device__ __forceinline__ int64_t tile_count(int uplo, int ntm, int ntn, int mt_m, int mt_n) {
    if (uplo == 0) return (int64_t)ntm * ntn;
    int64_t nt = 0;
    for (int first = 0; first < ntm; first += GROUP_M) {
        const int gsz = (ntm - first) < GROUP_M ? (ntm - first) : GROUP_M;
        nt += band_size(uplo, first, gsz, ntn, mt_m, mt_n);
    }
    return nt;
}

// Position of workgroup `bid` of `nt` in the tile order: the XCD that gets the workgroups bid = x (mod 8) owns
// one contiguous run of the order.
static __host__ __device__ __forceinline__ int lin_of_block(int bid, int nt) {
    const int per = (nt + NUM_XCD - 1) / NUM_XCD;
    int tall = nt % NUM_XCD;
    if (tall == 0) tall = NUM_XCD;
    const int xcd = bid % NUM_XCD, loc = bid / NUM_XCD;
    return xcd < tall ? xcd * per + loc : tall * per + (xcd - tall) * (per - 1) + loc;
}

// Tile at position `lin` of the tile order (bands of GROUP_M tile-rows, walked
// column by column).
struct TilePos { int tm, tn; };
static __host__ __device__ __forceinline__ TilePos tile_of_lin(int lin, int ntm, int ntn, int uplo, int mt_m,
                                                               int mt_n) {
    if (uplo == 0) {
        const int width = GROUP_M * ntn;
        const int grp = lin / width;
        const int first = grp * GROUP_M;
        const int gsz = (ntm - first) < GROUP_M ? (ntm - first) : GROUP_M;
        const int in = lin - grp * width;
        return TilePos{first + in % gsz, in / gsz};
    }
    // triangular: bands differ in size; walk them (uniform, scalar work)
    int first = 0;
    for (; first + GROUP_M < ntm; first += GROUP_M) {
        const int sz = band_size(uplo, first, GROUP_M, ntn, mt_m, mt_n);
        if (lin < sz) break;
        lin -= sz;
    }
    const int gsz = (ntm - first) < GROUP_M ? (ntm - first) : GROUP_M;
    const Band b = band_of(uplo, first, gsz, ntn, mt_m, mt_n);
    const int whole = gsz * (b.w1 - b.w0);
    if (uplo == 1) {
        if (lin < whole) return TilePos{first + lin % gsz, b.w0 + lin / gsz};
        lin -= whole;
    }
    for (int tn = b.p0; tn < b.p1; ++tn) {
        const ColRows c = col_rows(uplo, first, gsz, tn, mt_m, mt_n);
        if (lin < c.cnt) return TilePos{c.r0 + lin, tn};
        lin -= c.cnt;
    }
    if (uplo == 2 && lin < whole) return TilePos{first + lin % gsz, b.w0 + lin / gsz};
    return TilePos{ntm, ntn};   // past the end of the order: no tile
}

// ---------------------------------------------------------------------------
// Tile configuration.
// ---------------------------------------------------------------------------
// PF_: slabs between the global loads of a slab and its use (1: loaded while the slab before it is multiplied;
// 2: one slab earlier still, in a second set of staging registers, for variants whose slab is shorter than a
// memory round trip).
template <typename T, int MT_M_, int MT_N_, int KT_, int WGM_, int WGN_, int OCC_, int PF_ = 1> struct TileCfg {
    using M = Mfma<T>;
    static constexpr int MT_M = MT_M_, MT_N = MT_N_, KT = KT_, WGM = WGM_, WGN = WGN_, OCC = OCC_, PF = PF_;
    static_assert(PF == 1 || PF == 2, "prefetch distance in slabs");
    static constexpr int NT = WGM * WGN * 64;
    static constexpr int WT_M = MT_M / WGM, WT_N = MT_N / WGN;
    static constexpr int TM = WT_M / M::MI, TN = WT_N / M::MI;
    static_assert(WT_M % M::MI == 0 && WT_N % M::MI == 0, "wave tile must be whole MFMA tiles");
    static_assert(KT % M::KI == 0, "slab depth must be whole MFMA depths");
    // LDS row strides.  A fragment read takes 16-byte pieces of four slab rows at
    // once (the four depth steps of a matrix instruction), each row a run of 16
    // (fp64) / 32 (fp32) consecutive elements; with the row stride a multiple of
    // 256 bytes the four runs start on the same bank, and the counters show what
    // that costs: bank-conflict cycles are 20 % of the LDS-active cycles of the
    // fp64 N,N product, half a cycle per matrix instruction of 64, all of it in
    // the shadow of the matrix pipe.  The
    // stride matters for the writes of K-contiguous slabs: the KT/V lanes that
    // hold one row-vector mn write V rows apart, and with a power-of-two stride
    // they would all hit the same banks.  With W = 128 B / sizeof(T) elements per
    // LDS cycle, a stride of MT + 16 bytes makes the W lanes served in one cycle
    // fall on W distinct banks once the lanes are dealt to (k-chunk, mn) pairs
    // as Stager::pos does.  MN-contiguous slabs keep stride MT.
    static constexpr int VEC16 = 16 / (int)sizeof(T);
    static constexpr int PADK = VEC16;   // 16 bytes: rows stay aligned for vector reads
    static constexpr int stride(int mt, bool kcontig) { return kcontig ? mt + PADK : mt; }
    // MFMA tiles of a wave are interleaved along m (and n): tile i = ib*VR + t
    // covers rows  wm0 + ib*VR*MI + VR*idx + t  (idx = lane's operand index), so
    // one LDS read of VR consecutive elements feeds VR tiles and the epilogue
    // touches VR consecutive rows of C per lane (16-byte accesses).
    static constexpr int vr(int tiles) { return tiles % VEC16 == 0 ? VEC16 : (tiles % 2 == 0 ? 2 : 1); }
    static constexpr int VRM = vr(TM), VRN = vr(TN);
    static constexpr size_t LDS_BYTES = 2 * (size_t)KT * (MT_M + MT_N + 2 * PADK) * sizeof(T);
};

template <typename T, typename Cfg, bool AK, bool BK, bool FAST, bool SPLIT = false>
__global__ void __launch_bounds__(Cfg::NT, Cfg::OCC) gemm_kernel(const GemmArgs<T> g) {
    using M = Mfma<T>;
    constexpr int MT_M = Cfg::MT_M, MT_N = Cfg::MT_N, KT = Cfg::KT, NT = Cfg::NT;
    constexpr int SA = Cfg::stride(MT_M, AK), SB = Cfg::stride(MT_N, BK), TM = Cfg::TM, TN = Cfg::TN;
    using StA = Stager<T, MT_M, KT, SA, NT, AK>;
    using StB = Stager<T, MT_N, KT, SB, NT, BK>;

    extern __shared__ __align__(16) unsigned char lds_raw[];
    T *const lds = reinterpret_cast<T *>(lds_raw);
    // [buffer][A slab | B slab]
    constexpr int BUF = KT * (SA + SB);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave % Cfg::WGM) * Cfg::WT_M;
    const int wn0 = (wave / Cfg::WGM) * Cfg::WT_N;

    // which tile, and (SPLIT) which piece of its K range
    int lin, piece = 0, npieces = 1;
    if constexpr (SPLIT) {
        const int bid = blockIdx.x;
        if (bid < g.ndp) {
            lin = lin_of_block(bid, g.ndp);
        } else {
            npieces = g.nsplit;
            lin = g.ndp + (bid - g.ndp) / npieces;
            piece = (bid - g.ndp) % npieces;
        }
    } else {
        if (g.kcut == 0) {
            lin = lin_of_block(blockIdx.x, (int)gridDim.x);
        } else {
            // Tiles of unequal depth: one contiguous run of the order per XCD would give the XCDs unequal
            // work, so the order is dealt to them in squares of 64 tiles (8 x 8 tiles of one band) in turn.
            // The grid is a whole number of rounds of such squares; positions past the order have no tile.
            const int x = blockIdx.x % NUM_XCD, loc = blockIdx.x / NUM_XCD, total = g.ntm * g.ntn;
            lin = ((loc / 64) * NUM_XCD + x) * 64 + (loc % 64);
            if (lin >= total) return;
            if (g.reverse) lin = total - 1 - lin;
        }
    }
    int tm, tn;
    if (!SPLIT && g.sub_count > 0) {
        // position among the quarter tiles: one contiguous run of them per XCD, so that the quarters of a
        // tile and its neighbours share that XCD's L2
        const int b = lin_of_block(blockIdx.x, (int)gridDim.x);
        const TilePos big = tile_of_lin(g.sub_base + (b >> 2), g.sub_ntm, g.sub_ntn, g.uplo, 2 * MT_M, 2 * MT_N);
        tm = 2 * big.tm + (b & 1);
        tn = 2 * big.tn + ((b >> 1) & 1);
    } else {
        const TilePos tp = tile_of_lin(lin, g.ntm, g.ntn, g.uplo, MT_M, MT_N);
        tm = tp.tm;
        tn = tp.tn;
    }
    if (tm >= g.ntm || tn >= g.ntn) return;   // cannot happen when the grid is tile_count() workgroups
    const int m0 = tm * MT_M, n0 = tn * MT_N;
    const int m_lim = g.m - m0, n_lim = g.n - n0;   // rows / cols of this tile inside C
    // Triangular output (rank-k updates of a symmetric matrix): tiles wholly in
    // the other triangle leave at once, tiles wholly inside run as usual, tiles
    // the diagonal crosses take the predicated epilogue with the triangle test.
    bool on_diagonal = false;
    if (g.uplo == 1) {
        if (m0 + MT_M - 1 < n0) return;
        on_diagonal = m0 < n0 + MT_N - 1;
    } else if (g.uplo == 2) {
        if (n0 + MT_N - 1 < m0) return;
        on_diagonal = n0 < m0 + MT_M - 1;
    }
    const bool edge = m_lim < MT_M || n_lim < MT_N;

    // K range of this workgroup: all of it, or piece `piece` of `npieces` in whole slabs
    int k_begin = 0, k_len = g.k;
    if constexpr (SPLIT) {
        if (npieces > 1) {
            const int nsl = (g.k + KT - 1) / KT, base = nsl / npieces, extra = nsl % npieces;
            const int s0 = piece * base + (piece < extra ? piece : extra);
            const int cnt = base + (piece < extra ? 1 : 0);
            k_begin = s0 * KT;
            k_len = (g.k - k_begin) < cnt * KT ? (g.k - k_begin) : cnt * KT;
        }
    } else if (g.kcut != 0) {
        const int d = ((g.kaxis ? n0 : m0) / g.kblk) * g.kblk;
        if (g.kcut == 1) {
            k_len = d;
        } else {
            k_begin = d + g.kblk;
            k_len = g.k - k_begin;
        }
        if (k_len <= 0) return;   // nothing to add to this tile
    }

    // slab origins at depth k_begin
    const int64_t am0 = g.a_panel ? (int64_t)(m0 / PACK_W) * g.a_panel + m0 % PACK_W : (int64_t)m0;   // where row m0 starts
    const int64_t bn0 = g.b_panel ? (int64_t)(n0 / PACK_W) * g.b_panel + n0 % PACK_W : (int64_t)n0;
    const T *pa = AK ? g.A + (int64_t)m0 * g.lda + k_begin : g.A + am0 + (int64_t)k_begin * g.lda;
    const T *pb = BK ? g.B + (int64_t)n0 * g.ldb + k_begin : g.B + bn0 + (int64_t)k_begin * g.ldb;
    const int64_t step_a = AK ? (int64_t)KT : (int64_t)KT * g.lda;
    const int64_t step_b = BK ? (int64_t)KT : (int64_t)KT * g.ldb;

    // Position of accumulator (tile j, tile i, register r) of this lane in C:
    //   row m0 + c_m(i), column n0 + c_n(j, r)   (see the interleaving in TileCfg)
    constexpr int VRM = Cfg::VRM, VRN = Cfg::VRN;
    const int mc = wm0 + VRM * M::d_col(lane);
    auto c_n = [&](int j, int r) { return wn0 + (j / VRN) * VRN * M::MI + VRN * M::d_row(lane, r) + (j % VRN); };
    const bool full_tile = m_lim >= MT_M && n_lim >= MT_N && !on_diagonal;
    const T alpha = g.alpha, beta = g.beta;
    typename M::acc_t acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < M::NR; ++r) acc[j][i][r] = T(0);

    constexpr int PF = Cfg::PF;
    typename StA::vec_t ra[PF][StA::NV];      // staging registers: set s holds the slabs t with t % PF == s
    typename StB::vec_t rb[PF][StB::NV];
    uint32_t offa[StA::NV], offb[StB::NV];
    StA::offsets(offa, g.lda, tid);
    StB::offsets(offb, g.ldb, tid);
    // Full-depth slabs go the 16-byte way on edge tiles too, with the vectors
    // outside the tile's rows and columns switched off.  A vector that straddles
    // the edge reads up to V - 1 elements past it; in the last stored column of
    // the operand those could lie past the end of the array, so with a straddle
    // a slab goes the fast way only while another column follows it (guard), and
    // not at all if the columns are shorter than a vector.
    bool hot = FAST;
    int guard = 0;
    if (FAST && edge) {
        StA::trim(offa, tid, m_lim);
        StB::trim(offb, tid, n_lim);
        if (StA::straddles(m_lim)) { guard = 1; hot = hot && g.lda >= StA::V; }
        if (StB::straddles(n_lim)) { guard = 1; hot = hot && g.ldb >= StB::V; }
    }

    const int nslab = (k_len + KT - 1) / KT;

    // slab t (the next one in order: pa, pb walk along K) into its set of staging registers; `set` is t % PF as a
    // constant at every call site
    auto fetch = [&](int t, int set) {
        const int k_lim = k_len - t * KT;
        if (hot && k_lim >= KT + guard) {
            StA::load_fast(ra[set], pa, offa);
            StB::load_fast(rb[set], pb, offb);
        } else if (FAST) {
            StA::load_edge(ra[set], pa, offa, tid, m_lim, k_lim);
            StB::load_edge(rb[set], pb, offb, tid, n_lim, k_lim);
        } else {
            StA::load_guarded(ra[set], pa, g.lda, tid, m_lim, k_lim);
            StB::load_guarded(rb[set], pb, g.ldb, tid, n_lim, k_lim);
        }
        pa += step_a;
        pb += step_b;
    };
    T *const stash_a = lds + StA::lds_origin(tid);
    T *const stash_b = lds + KT * SA + StB::lds_origin(tid);
    auto stash = [&](int buf, int set) {
        StA::store(ra[set], stash_a + buf * BUF);
        StB::store(rb[set], stash_b + buf * BUF);
    };

    // Operand fragments are double-buffered in registers: the LDS reads of
    // MFMA group g+1 are issued before the MFMAs of group g, so a read has a whole
    // group of MFMAs to land (the paper's rule of giving each permutation of b its
    // own register so that loads never wait on the compute that still uses the
    // old value, Sec. 5.2).
    constexpr int NG = KT / M::KI;   // MFMA groups (rank-KI updates of the wave tile) per slab
    static_assert(NG % 2 == 0, "fragment double buffering needs an even number of groups per slab");
    const int kq = M::op_k(lane), iq = M::op_idx(lane);
    const T *const frag_a = lds + kq * SA + wm0 + VRM * iq;
    const T *const frag_b = lds + KT * SA + kq * SB + wn0 + VRN * iq;
    T fa[2][TM], fb[2][TN];
    // buf, grp and set are compile-time constants at every call site, so each
    // read is "per-lane base register + immediate offset".
    auto load_frags = [&](int buf, int grp, int set) {
        const T *sa = frag_a + buf * BUF + grp * M::KI * SA;
        const T *sb = frag_b + buf * BUF + grp * M::KI * SB;
#pragma unroll
        for (int ib = 0; ib < TM / VRM; ++ib) {
            T v[VRM];
            Pack<T, VRM>::load(sa + ib * VRM * M::MI, v);
#pragma unroll
            for (int u = 0; u < VRM; ++u) fa[set][ib * VRM + u] = v[u];
        }
#pragma unroll
        for (int jb = 0; jb < TN / VRN; ++jb) {
            T v[VRN];
            Pack<T, VRN>::load(sb + jb * VRN * M::MI, v);
#pragma unroll
            for (int u = 0; u < VRN; ++u) fb[set][jb * VRN + u] = v[u];
        }
    };
    auto mma_group = [&](int set) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int i = 0; i < TM; ++i) acc[j][i] = M::mma(fb[set][j], fa[set][i], acc[j][i]);
    };

    // ramp-up: slab 0 into LDS buffer 0, first fragments into registers
    fetch(0, 0);
    stash(0, 0);
    if constexpr (PF == 2) {
        if (nslab > 1) fetch(1, 1);
    }
    __syncthreads();
    load_frags(0, 0, 0);

    // steady state.  Per slab t (LDS buffer cur = t & 1): global loads of slab
    // t+1 go out first; MFMA groups 0..NG-2 run with the next group's fragments
    // in flight; then slab t+1 is written to the other LDS buffer and the
    // workgroup synchronises; the last MFMA group of slab t is issued AFTER the
    // barrier, together with the first fragment reads of slab t+1, so the
    // post-barrier LDS latency is covered by a full group of MFMAs.
    // (the LDS buffer of slab t is t & 1 = cur; with PF == 2 that is also its set of staging registers, and the
    // slab asked for here is t + 2, into the set that slab t has left)
    auto slab = [&](int t, int cur) {
        const bool more = (t + 1 < nslab);
        if constexpr (PF == 2) {
            if (t + 2 < nslab) fetch(t + 2, cur);
        } else {
            if (more) fetch(t + 1, 0);
        }
#pragma unroll
        for (int grp = 0; grp + 1 < NG; ++grp) {
            load_frags(cur, grp + 1, (grp + 1) & 1);
            mma_group(grp & 1);
        }
        if (more) stash(cur ^ 1, PF == 2 ? cur ^ 1 : 0);
        __syncthreads();
        if (more) load_frags(cur ^ 1, 0, 0);
        mma_group((NG - 1) & 1);
    };
    // The same step with nothing to decide: the tile is interior and the next
    // slab is a full one, so the body is straight-line code (one scheduling
    // region per pair of slabs).
    // Instruction classes for the scheduler hints below.
    constexpr int SG_MFMA = 0x008, SG_VMEM_RD = 0x020, SG_DS_RD = 0x100, SG_DS_WR = 0x200;
    constexpr int N_MMA = TM * TN;                       // MFMAs per group
    constexpr int N_FRAG = TM / VRM + TN / VRN;          // LDS reads per group
    constexpr int N_LD = StA::NV + StB::NV;              // global loads per slab
    constexpr int N_ST = (AK ? StA::NV * StA::V : StA::NV) + (BK ? StB::NV * StB::V : StB::NV);   // LDS writes (upper bound)
    auto slab_hot = [&](int cur) {
        StA::load_fast(ra[PF == 2 ? cur : 0], pa, offa);      // slab t + PF
        StB::load_fast(rb[PF == 2 ? cur : 0], pb, offb);
        pa += step_a;
        pb += step_b;
#pragma unroll
        for (int grp = 0; grp + 1 < NG; ++grp) {
            load_frags(cur, grp + 1, (grp + 1) & 1);
            mma_group(grp & 1);
        }
        stash(cur ^ 1, PF == 2 ? cur ^ 1 : 0);
        // schedule of the region that ends at the barrier: global loads under
        // the first MFMAs, each group's fragment reads under its predecessor,
        // LDS writes under the last MFMAs before the barrier
        constexpr int PRE = (NG - 1) * N_MMA;        // MFMAs before the barrier
        constexpr int N_RD = (NG - 1) * N_FRAG;      // fragment reads before the barrier
        constexpr int Q = shadow_quota(PRE, N_LD, N_RD, N_ST);
        constexpr int Q2 = shadow_quota(N_MMA, 0, N_FRAG, 0);
        constexpr bool HINT = Q > 0 && Q2 > 0;
        if constexpr (HINT) {
            interleave<SG_VMEM_RD, N_LD, Q>();
            interleave<SG_DS_RD, N_RD, Q>();
            constexpr int REST = PRE - ceil_div(N_LD, Q) - ceil_div(N_RD, Q) - ceil_div(N_ST, Q);
            if constexpr (REST > 0) __builtin_amdgcn_sched_group_barrier(SG_MFMA, REST, 0);
            interleave<SG_DS_WR, N_ST, Q>();
        }
        __syncthreads();
        load_frags(cur ^ 1, 0, 0);
        mma_group((NG - 1) & 1);
        if constexpr (HINT) {
            interleave<SG_DS_RD, N_FRAG, Q2>();
            constexpr int REST2 = N_MMA - ceil_div(N_FRAG, Q2);
            if constexpr (REST2 > 0) __builtin_amdgcn_sched_group_barrier(SG_MFMA, REST2, 0);
        }
    };
    // Two slabs per trip so that the LDS buffer index is a constant in the code.
    int t = 0;
    if (hot) {
        const int nfull = (k_len - guard) / KT;   // slabs 0..nfull-1 are full (and, with a straddle, not the last column)
        for (; t + 1 + PF < nfull; t += 2) {
            slab_hot(0);
            slab_hot(1);
        }
        if (t + PF < nfull) {   // one more slab whose successor (second successor) is full
            slab_hot(0);
            ++t;
        }
    }
    if (t & 1) {
        slab(t, 1);
        ++t;
    }
    for (; t < nslab; t += 2) {
        slab(t, 0);
        if (t + 1 < nslab) slab(t + 1, 1);
    }

    // flush of one accumulator row-block j (the MFMA tiles (j, 0..TM-1) of this
    // wave): C = alpha*acc + beta*C on the part of the tile inside C
    const bool use_c = (beta != T(0));
    // whole tile inside C: no predicates, 16-byte accesses.  The reads of C of a
    // row-block are issued together ahead of the first dependent store, so each
    // row-block costs one memory round trip.
    auto flush_full = [&](int j, const typename M::acc_t (&a)[TM]) {
        T *cp[M::NR];
        T cold[M::NR][TM];
#pragma unroll
        for (int r = 0; r < M::NR; ++r) cp[r] = g.C + (int64_t)(n0 + c_n(j, r)) * g.ldc + m0 + mc;
        if (use_c) {
#pragma unroll
            for (int r = 0; r < M::NR; ++r)
#pragma unroll
                for (int ib = 0; ib < TM / VRM; ++ib) {
                    T v[VRM];
                    Pack<T, VRM>::load(cp[r] + ib * VRM * M::MI, v);
#pragma unroll
                    for (int u = 0; u < VRM; ++u) cold[r][ib * VRM + u] = v[u];
                }
        }
#pragma unroll
        for (int r = 0; r < M::NR; ++r)
#pragma unroll
            for (int ib = 0; ib < TM / VRM; ++ib) {
                T v[VRM];
#pragma unroll
                for (int u = 0; u < VRM; ++u) {
                    v[u] = alpha * a[ib * VRM + u][r];
                    if (use_c) v[u] += beta * cold[r][ib * VRM + u];
                }
                Pack<T, VRM>::store(cp[r] + ib * VRM * M::MI, v);
            }
    };
    // edge or diagonal tile: element by element under the bounds and triangle tests
    // The elements are addressed from the tile's origin through a range-checked buffer: one that lies outside C or
    // outside the triangle gets an offset beyond the range, reads as zero and is not written, so a row-block is
    // one batch of loads and one batch of stores with no branch between them (a branch per element made the
    // compiler wait for each element's round trip in turn).  Leading dimensions too large for 31-bit offsets
    // inside a tile take the element-by-element way.
    const bool c_in_range = (int64_t)g.ldc * (int64_t)(MT_N * sizeof(T)) < (int64_t)0x7fffffff;
    auto flush_edge = [&](int j, const typename M::acc_t (&a)[TM]) {
        if (c_in_range) {
            constexpr uint32_t OUTSIDE = 0x80000000u;
            const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(g.C + (int64_t)n0 * g.ldc + m0, 0, (int)OUTSIDE, 0x00020000);
            // RB accumulator registers (columns of C) at a time: at most 16 elements per lane in flight,
            // so that the offsets and the old values never push a variant over its register budget
            constexpr int RB = (16 / TM > 0) ? ((16 / TM < M::NR) ? 16 / TM : M::NR) : 1;
            static_assert(M::NR % RB == 0, "row-blocks are flushed in whole batches");
#pragma unroll
            for (int r0 = 0; r0 < M::NR; r0 += RB) {
                uint32_t off[RB][TM];
#pragma unroll
                for (int r = 0; r < RB; ++r) {
                    const int nn = c_n(j, r0 + r);
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const int mm = mc + (i / VRM) * VRM * M::MI + (i % VRM);
                        const int below = (g.uplo == 2) ? (n0 - m0) + nn - mm : (m0 - n0) + mm - nn;
                        const bool ok = mm < m_lim && nn < n_lim && (g.uplo == 0 || below >= 0);
                        off[r][i] = ok ? (uint32_t)(((int64_t)nn * g.ldc + mm) * (int64_t)sizeof(T)) : OUTSIDE;
                    }
                }
                T cold[RB][TM];
                if (use_c) {
#pragma unroll
                    for (int r = 0; r < RB; ++r)
#pragma unroll
                        for (int i = 0; i < TM; ++i) {
                            if constexpr (sizeof(T) == 8) {
                                typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
                                cold[r][i] = __builtin_bit_cast(T, (u32x2)__builtin_amdgcn_raw_buffer_load_b64(rc, off[r][i], 0, 0));
                            } else {
                                cold[r][i] = __builtin_bit_cast(T, (unsigned int)__builtin_amdgcn_raw_buffer_load_b32(rc, off[r][i], 0, 0));
                            }
                        }
                }
#pragma unroll
                for (int r = 0; r < RB; ++r)
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        T v = alpha * a[i][r0 + r];
                        if (use_c) v += beta * cold[r][i];
                        if constexpr (sizeof(T) == 8) {
                            typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
                            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), rc, off[r][i], 0, 0);
                        } else {
                            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), rc, off[r][i], 0, 0);
                        }
                    }
            }
            return;
        }
#pragma unroll
        for (int r = 0; r < M::NR; ++r) {
            const int nn = c_n(j, r);
            T *crow = g.C + (int64_t)(n0 + nn) * g.ldc + m0;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int mm = mc + (i / VRM) * VRM * M::MI + (i % VRM);
                // signed distance below the diagonal, flipped for the upper triangle
                const int below = (g.uplo == 2) ? (n0 - m0) + nn - mm : (m0 - n0) + mm - nn;
                if (mm < m_lim && nn < n_lim && (g.uplo == 0 || below >= 0)) {
                    T v = alpha * a[i][r];
                    if (use_c) v += beta * crow[mm];
                    crow[mm] = v;
                }
            }
        }
    };

    // Split tile: leave the partial sums in the workspace (in register order, so
    // every store covers NT consecutive vectors); the piece that arrives last
    // adds all of them in a fixed order, which makes the result independent of
    // the order of arrival, and flushes.  Nobody waits for anybody.
    // The partial sums travel between compute units that may sit on different
    // XCDs, whose L2 caches are not coherent with each other: they are written
    // through to memory and read around the caches (system-scope accesses), so
    // that no cache has to be flushed or invalidated as a whole; the arrival
    // counter is a device-scope atomic issued after this workgroup's stores have
    // been acknowledged.
    if constexpr (SPLIT) {
        if (npieces > 1) {
            typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
            typedef typename StA::vec_t vec_t;
            constexpr int PV = Cfg::VEC16;                         // registers per 16-byte access
            constexpr int THROUGH = 17;                            // cache policy bits sc0 | sc1
            static_assert(M::NR % PV == 0, "accumulator registers must pack into 16-byte vectors");
            constexpr int64_t TILE = (int64_t)MT_M * MT_N;
            constexpr int NVJ = TM * M::NR / PV;                   // 16-byte vectors of one row-block
            const int q = lin - g.ndp;                             // index of the split tile
            const uint32_t lane_off = (uint32_t)tid * 16u;
            {
                const __amdgpu_buffer_rsrc_t mine = __builtin_amdgcn_make_buffer_rsrc(
                    g.part + ((int64_t)q * npieces + piece) * TILE, 0, (int)(TILE * sizeof(T)), 0x00020000);
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int r = 0; r < M::NR; r += PV) {
                            vec_t v;
#pragma unroll
                            for (int u = 0; u < PV; ++u) v[u] = acc[j][i][r + u];
                            const int vi = j * NVJ + (i * M::NR + r) / PV;
                            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), mine,
                                                                   lane_off + (uint32_t)vi * (NT * 16u), 0, THROUGH);
                        }
            }
            // every store of this wave acknowledged (vmcnt(0); the other counters stay as they are)
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            unsigned *const flag = reinterpret_cast<unsigned *>(lds_raw);
            if (tid == 0) *flag = __hip_atomic_fetch_add(g.cnt + q, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (*flag != (unsigned)(npieces - 1)) return;
            // leave the counter as it was found
            if (tid == 0) __hip_atomic_store(g.cnt + q, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // row-block by row-block: sum of the pieces in the order 0, 1, ..., then flush
            const T *const tile0 = g.part + (int64_t)q * npieces * TILE;
#pragma unroll 1
            for (int j = 0; j < TN; ++j) {
                typename M::acc_t sum[TM];
#pragma unroll 1
                for (int sp = 0; sp < npieces; ++sp) {
                    const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(
                        const_cast<T *>(tile0 + (int64_t)sp * TILE), 0, (int)(TILE * sizeof(T)), 0x00020000);
                    vec_t v[NVJ];
#pragma unroll
                    for (int vi = 0; vi < NVJ; ++vi)
                        v[vi] = __builtin_bit_cast(vec_t, (u32x4)__builtin_amdgcn_raw_buffer_load_b128(
                                                              src, lane_off + (uint32_t)(j * NVJ + vi) * (NT * 16u), 0,
                                                              THROUGH));
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int r = 0; r < M::NR; r += PV)
#pragma unroll
                            for (int u = 0; u < PV; ++u) {
                                const T x = v[(i * M::NR + r) / PV][u];
                                sum[i][r + u] = (sp == 0) ? x : sum[i][r + u] + x;
                            }
                }
                if (full_tile) flush_full(j, sum);
                else flush_edge(j, sum);
            }
            return;
        }
    }

    if (full_tile) {
#pragma unroll
        for (int j = 0; j < TN; ++j) flush_full(j, acc[j]);
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) flush_edge(j, acc[j]);
    }
}

// C := beta * C (beta == 0 stores zeros without reading), the alpha == 0 / k == 0 path;
// uplo as in GemmArgs.
template <typename T>
__global__ void __launch_bounds__(256) scale_kernel(T *C, int64_t ldc, int m, int n, T beta, int uplo) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= m) return;
    for (int j = blockIdx.y; j < n; j += gridDim.y) {
        if ((uplo == 1 && i < j) || (uplo == 2 && i > j)) continue;
        T *p = C + i + (int64_t)j * ldc;
        *p = (beta == T(0)) ? T(0) : beta * *p;
    }
}

}  // namespace xg
