// Host side of libdgsp: argument checks, launch geometry, the selector.
// The C-ABI is documented in include/dgsp.h.
#include "../../include/dgsp.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <map>
#include <mutex>
#include <utility>

#include "dgsp_kernels.hpp"

namespace {

using namespace dgsp;

// ---------------------------------------------------------------- device facts
struct DeviceInfo {
    int cus = 0;
};

DeviceInfo device_info() {
    static std::mutex mu;
    static DeviceInfo cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return DeviceInfo{256};
    std::lock_guard<std::mutex> lock(mu);
    if (cache[dev].cus == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        cache[dev].cus = cus;
    }
    return cache[dev];
}

inline int ilog2_ceil(long long v) {   // smallest l with 2^l >= v  (v >= 1)
    int l = 0;
    while ((1LL << l) < v) ++l;
    return l;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline unsigned clamp_blocks(long long want, long long cap) {
    if (want < 1) want = 1;
    return (unsigned)(want < cap ? want : cap);
}

// resident waves per CU assumed when sizing machine-filling grids
constexpr int kBlocksPerCu = 8;

static_assert((1 << kNbSrLogTile) == kNbSrTile, "tile must be a power of two");

// Rows count as "about equally long" for the launch geometry of the row-split sequential kernel when the
// caller's statistics give a coefficient of variation up to this (a property of the kernel's schedule, fixed
// here; the selector's thresholds are separate state and do not reach the launch code).
constexpr double kEvenRowsCvMax = 0.3;
// largest leading dimension of Y the balanced kernels take (a tile's rows are stored through 32-bit byte offsets)
constexpr int64_t kBalancedLdyMax = 1 << 20;

// What a caller's row statistics tell the launch code (nothing, when it passed none).
struct Hints {
    double col_span = 0.0;
    double cv_row = -1.0;
    Hints() = default;
    explicit Hints(const dgsp_features_t* f) { if (f) { col_span = f->col_span; cv_row = f->cv_row; } }
};

struct Problem {
    int M, N;
    int ldx, ldy;       // leading dimensions of X and Y in elements (>= N)
    long long K, nnz;   // nnz < 0: unknown on the host
    const int* rowptr; const int* colidx; const float* vals; const float* X; float* Y;
    hipStream_t stream;
    int phase = DGSP_PHASE_ALL;
    double col_span = 0.0;   // mean column span of a row / K; 0 = unknown
    double cv_row = -1.0;    // coefficient of variation of the row lengths; < 0 = unknown
    int switches = 0;        // DGSP_ABL_* (measurement aids)
    bool scaled = false;     // Y = alpha * A X + beta * Y instead of Y = A X
    float alpha = 1.0f, beta = 0.0f;
};

// Vector width of the comparison kernel without LDS staging (rs_sr_direct_kernel) only: it uses plain
// float2 / float4 accesses, which need N, the leading dimensions and the addresses of X and Y to fit.
// The four kernels proper do not depend on alignment (see pr_vector_width, sr_shape).
inline int direct_kernel_vector_width(const Problem& p) {
    if (p.switches & DGSP_ABL_SCALAR_DENSE_LOADS) return 1;
    int v = 1;
    if (p.N % 4 == 0 && aligned(p.X, 16) && aligned(p.Y, 16)) v = 4;
    else if (p.N % 2 == 0 && aligned(p.X, 8) && aligned(p.Y, 8)) v = 2;
    while (v > 1 && (p.ldx % v != 0 || p.ldy % v != 0)) v >>= 1;     // every row must start aligned
    return v;
}

// Dense columns per lane and pass of the parallel-reduction kernels: the widest of 4, 3, 2 that divides N (one
// dwordx4 / x3 / x2 access, taken at any dword address, so alignment and leading dimensions do not matter).
inline int pr_vector_width(int64_t N, int switches) {
    if (switches & DGSP_ABL_SCALAR_DENSE_LOADS) return 1;
    return N % 4 == 0 ? 4 : N % 3 == 0 ? 3 : N % 2 == 0 ? 2 : 1;
}
inline int pr_vector_width(const Problem& p) { return pr_vector_width(p.N, p.switches); }
// The same for the balanced parallel kernel, which also has eight columns per lane (two dwordx4 accesses): when 8
// divides N - one pass over A instead of two - and for N = 5, 6, 7 with the two groups of four overlapping.
inline int nb_pr_lane_width(int64_t N, int switches) {
    const int v = pr_vector_width(N, switches);
    if (v == 4 && N % 8 == 0) return 8;
    if (N >= 5 && N <= 7 && !(switches & DGSP_ABL_SCALAR_DENSE_LOADS)) return 8;
    return v;
}

#define DGSP_LAUNCH(kernel, grid, ...)                                                        \
    do {                                                                                      \
        hipLaunchKernelGGL(kernel, grid, dim3(kBlock), 0, p.stream, __VA_ARGS__);             \
        if (hipGetLastError() != hipSuccess) return DGSP_ERR_LAUNCH;                          \
    } while (0)

// ---------------------------------------------------------------- launch geometry helpers
// Workgroups of `kernel` that one CU keeps resident (registers and LDS decide).  The balanced
// kernels cut the work into equal shares per wave, so their grid must not exceed what runs at
// once: a workgroup that waits for a slot would start its share when the others are done.
template <typename K>
int resident_blocks_per_cu(K kernel) {
    static std::mutex mu;
    static std::map<std::pair<const void*, int>, int> cache;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 4;
    const auto key = std::make_pair(reinterpret_cast<const void*>(kernel), dev);
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find(key);
    if (it != cache.end()) return it->second;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, kBlock, 0) != hipSuccess || n <= 0) n = 4;
    cache[key] = n;
    return n;
}

// ---------------------------------------------------------------- row-split launches
// X can be addressed with 32-bit byte offsets (through a buffer descriptor)
constexpr unsigned long long kL2BytesPerXcd = 4ull << 20;      // gfx950: 4 MB of L2 per XCD

inline bool x_fits_descriptor(const Problem& p) {
    return dense_bytes(p.K, p.ldx, p.N) <= 0xffffffffull;
}

template <int V, bool XBUF>
int launch_rs_pr_v(const Problem& p) {
    const int logG = p.nnz >= 0 ? pr_lanes_log2(p.nnz, p.M) : -1;
    // one wave per row group when lanes-per-row is known; else assume the
    // finest split the kernel may choose (2 lanes per row) and let waves stride
    const int rows_per_wave = (kWave >> (logG >= 0 ? logG : 1)) * kRsPrUnroll;
    const long long groups = ((long long)p.M + rows_per_wave - 1) / rows_per_wave;
    const long long cap = (long long)device_info().cus * kBlocksPerCu * 8;
    const dim3 grid(clamp_blocks((groups + kWavesPerBlock - 1) / kWavesPerBlock, cap));
    if (p.scaled) {
        DGSP_LAUNCH((rs_pr_kernel<V, XBUF, true>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X,
                    p.Y, logG, Scaling{p.alpha, p.beta});
        return DGSP_OK;
    }
    DGSP_LAUNCH((rs_pr_kernel<V, XBUF>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X, p.Y, logG);
    return DGSP_OK;
}

int launch_rs_pr(const Problem& p) {
    const bool xb = x_fits_descriptor(p);
    switch (pr_vector_width(p)) {
        case 4: return xb ? launch_rs_pr_v<4, true>(p) : launch_rs_pr_v<4, false>(p);
        case 3: return xb ? launch_rs_pr_v<3, true>(p) : launch_rs_pr_v<3, false>(p);
        case 2: return xb ? launch_rs_pr_v<2, true>(p) : launch_rs_pr_v<2, false>(p);
        default: return xb ? launch_rs_pr_v<1, true>(p) : launch_rs_pr_v<1, false>(p);
    }
}

// lanes per row of the sequential kernels: enough lanes of width V to span N, at most a wave
inline int sr_lanes_log2(long long N, int V, int cap = 6) {
    const long long need = (N + V - 1) / V;
    const int lg = ilog2_ceil(need);
    return lg > cap ? cap : lg;
}

// Column blocks of the sequential kernels.  A group of G lanes (a power of two) walks the entries once per block,
// so a call costs about blocks * G lane-steps per entry, and every further pass over the matrix costs more than
// its share (measured +15 ... +33 % per extra pass at equal blocks * G).  The blocks are made equally wide (three
// blocks for N = 300 are 100 + 100 + 100, not 128 + 128 + 44).  `narrow`: N is a multiple of 64 and the caller
// wants blocks of 64 columns, all lanes busy in every block (see the launch functions for when that pays).
struct SrColumns { int logG; int cols_per_block; unsigned blocks; };
inline SrColumns sr_columns(long long N, int V, bool narrow) {
    const long long lanes = (N + V - 1) / V;
    long long blocks = 1;
    if (narrow && N % 64 == 0) {
        blocks = N / 64;
    } else {
        double best = 0.0;
        for (int lg = 0; lg <= 6; ++lg) {
            const long long b = (lanes + (1ll << lg) - 1) >> lg;
            const double cost = (double)(b << lg) * (1.0 + 0.3 * (double)(b - 1));
            if (lg == 0 || cost <= best) { best = cost; blocks = b; }         // ties: the wider group, fewer passes
        }
    }
    const long long per = (((N + blocks - 1) / blocks + V - 1) / V) * V;        // a multiple of V
    return {sr_lanes_log2(per, V), (int)per, (unsigned)((N + per - 1) / per)};
}

// Dense-row loads in flight per lane of the sequential kernels: enough to fill, not to overflow,
// the L1 when rows of X are scattered (about 1 KB per wave: 4 / V loads), four when the matrix is
// known to be banded (neighbouring rows then share their rows of X and mostly hit in cache).
inline bool banded(const Problem& p) { return p.col_span > 0.0 && p.col_span <= 0.05; }

// The sequential kernels give a lane four dense columns whenever a row has four: the memory pipeline takes
// dwordx2 / dwordx4 accesses at any dword address, so neither the alignment of X and Y nor their leading
// dimensions restrict the width.  When N is not a multiple of four the last lane of a row takes the row's last
// four columns; those it shares with its neighbour are the neighbour's to add or to scale (RAGGED).
struct SrShape { int v; bool ragged; };
inline SrShape sr_shape(const Problem& p) {
    if (p.switches & DGSP_ABL_SCALAR_DENSE_LOADS) return {1, false};
    // N = 3 and N = 6 keep the widest width that divides them: so few columns do not repay the extra stores
    // of the shared lane (measured: +6 % at N = 6, +7 ... +17 % at N = 3 with it; N = 5 gains 13 %, N = 7 is even)
    if (p.N == 3) return {1, false};
    if (p.N == 6 || p.N == 2) return {2, false};
    const int v = p.N >= 4 ? 4 : 1;
    return {v, p.N % v != 0};
}
// dense-row loads in flight per lane (see banded())
template <int V> constexpr int sr_depth_scattered() { return V == 4 ? 1 : V == 2 ? 2 : 4; }

template <int V, bool XBUF, int DEPTH, bool RAGGED>
int launch_rs_sr_v(const Problem& p) {
    // Rows of about equal length (what the selection rules send here) and N a multiple of 64: column blocks of 64
    // dense columns as in the balanced kernel, four rows per wave in step; 2-16 % faster at N >= 128 on such matrices.
    // With long rows among short ones the rows of a wave wait for the longest (+30 % measured), and without row
    // statistics nothing is known: then a group spans the whole width.
    const bool even_rows = p.cv_row >= 0.0 && p.cv_row <= kEvenRowsCvMax;
    const SrColumns cols = sr_columns(p.N, V, even_rows && p.N >= 128);
    const int logG = cols.logG;
    const unsigned col_blocks = cols.blocks;
    if (col_blocks > 65535u) return DGSP_ERR_INVALID_ARG;
    const int rows_per_wave = kWave >> logG;
    const long long groups = ((long long)p.M + rows_per_wave - 1) / rows_per_wave;
    const long long cap = (long long)device_info().cus * kBlocksPerCu * 8;
    const dim3 grid(clamp_blocks((groups + kWavesPerBlock - 1) / kWavesPerBlock, cap), col_blocks);
    if (p.scaled) {
        DGSP_LAUNCH((rs_sr_kernel<V, XBUF, DEPTH, true, RAGGED>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals,
                    p.X, p.Y, logG, cols.cols_per_block, Scaling{p.alpha, p.beta});
        return DGSP_OK;
    }
    DGSP_LAUNCH((rs_sr_kernel<V, XBUF, DEPTH, false, RAGGED>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X,
                p.Y, logG, cols.cols_per_block);
    return DGSP_OK;
}

template <int V>
int launch_rs_sr_direct_v(const Problem& p) {
    // the same column blocks as the kernel it is compared with
    const bool even_rows = p.cv_row >= 0.0 && p.cv_row <= kEvenRowsCvMax;
    const SrColumns cols = sr_columns(p.N, V, even_rows && p.N >= 128);
    const int logG = cols.logG;
    const unsigned col_blocks = cols.blocks;
    if (col_blocks > 65535u) return DGSP_ERR_INVALID_ARG;
    const int rows_per_wave = kWave >> logG;
    const long long groups = ((long long)p.M + rows_per_wave - 1) / rows_per_wave;
    const long long cap = (long long)device_info().cus * kBlocksPerCu * 8;
    const dim3 grid(clamp_blocks((groups + kWavesPerBlock - 1) / kWavesPerBlock, cap), col_blocks);
    DGSP_LAUNCH((rs_sr_direct_kernel<V>), grid, p.M, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X, p.Y, logG,
                cols.cols_per_block);
    return DGSP_OK;
}

template <int V, bool RAGGED>
int launch_rs_sr_pick(const Problem& p) {
    const bool xb = x_fits_descriptor(p);
    // X inside one XCD's L2: nothing to keep together, so hide latency with four loads in flight (-9 % on
    // Poisson(16) rows, -37 % on rows of 64 at N = 4, 2^18 rows).  Beyond that size the single load is what
    // keeps the lanes of a wave in step over the same part of X (four in flight: +10 ... +70 % there).
    if (banded(p) || dense_bytes(p.K, p.ldx, p.N) <= kL2BytesPerXcd)
        return xb ? launch_rs_sr_v<V, true, 4, RAGGED>(p) : launch_rs_sr_v<V, false, 4, RAGGED>(p);
    constexpr int D = sr_depth_scattered<V>();
    return xb ? launch_rs_sr_v<V, true, D, RAGGED>(p) : launch_rs_sr_v<V, false, D, RAGGED>(p);
}

int launch_rs_sr(const Problem& p) {
    if (p.switches & DGSP_ABL_NO_SPARSE_STAGING) {
        switch (direct_kernel_vector_width(p)) {
            case 4: return launch_rs_sr_direct_v<4>(p);
            case 2: return launch_rs_sr_direct_v<2>(p);
            default: return launch_rs_sr_direct_v<1>(p);
        }
    }
    const SrShape shape = sr_shape(p);
    switch (shape.v) {
        case 4: return shape.ragged ? launch_rs_sr_pick<4, true>(p) : launch_rs_sr_pick<4, false>(p);
        case 2: return launch_rs_sr_pick<2, false>(p);
        default: return launch_rs_sr_pick<1, false>(p);
    }
}

// ---------------------------------------------------------------- balanced launches
// Zeroes (scaled form: multiplies by beta) the rows split by the `parts` chunks the main kernel derives
// (quanta of 2^quantum_log2 items), cut into tiles of 2^tile_log2 items (tile_log2 < 0: not cut further).
int launch_prepare(const Problem& p, unsigned parts, unsigned quantum_log2, int tile_log2) {
    const dim3 grid((unsigned)(((long long)p.M + kBlock - 1) / kBlock));
    DGSP_LAUNCH(nb_prepare_kernel, grid, p.M, p.N, p.ldy, p.rowptr, p.Y, parts, quantum_log2, tile_log2,
                p.scaled ? p.beta : 0.0f);
    return DGSP_OK;
}

// Blocks of the grid that shares the nnz + M merge-path items of a balanced kernel, `tile` items per
// tile.  The gathers of a CU go through one L1 whose capacity for outstanding misses bounds them,
// whatever the number of waves, so CUs must finish together: the grid is a whole multiple of the CU
// count (544 blocks on 256 CUs ran 25 % slower than 512).  A matrix too small for one tile per wave
// on every CU gets one wave per tile.  Blocks per CU, at most what is resident:
//   sequential kernel: as many as there are tiles for (its dense-row loads want every wave they can get);
//   parallel kernel: one per 12 tiles per wave - a wave pays a start-up (a search in rowptr, loads
//     that nothing overlaps yet) and fewer waves leave more of the L1 to each - but two as soon as
//     that leaves a wave 6 tiles (measured on matrices of 1 M to 57 M entries).
constexpr long long kNbPrTilesPerWave = 12;
// quads of entries per lane and tile / block in the balanced parallel kernel for up to four columns per lane
// (four quads, 1024 items: 4-8 % faster on the stencil with item tiles, 2-12 % slower with entry blocks and on R-MAT)
constexpr int kNbPrKq = 2;

inline unsigned balanced_blocks(const Problem& p, long long tile, int blocks_per_cu, bool parallel,
                                long long col_blocks = 1, long long parallel_per_cu_max = 0) {
    const long long cus = device_info().cus;
    const long long cap = cus * blocks_per_cu;
    // entry count unknown on the host (the 10-argument call): what serves large matrices best
    if (p.nnz < 0) return (unsigned)(parallel && blocks_per_cu > 2 ? cus * 2 : cap);
    const long long tiles = (p.nnz + p.M + tile - 1) / tile;
    const long long waves = cus * kWavesPerBlock;
    if (tiles <= waves) return clamp_blocks((tiles + kWavesPerBlock - 1) / kWavesPerBlock, cap);
    long long per_cu;
    if (parallel) {
        per_cu = tiles / (waves * kNbPrTilesPerWave);
        if (per_cu < 2) per_cu = tiles >= waves * kNbPrTilesPerWave ? 2 : 1;
        if (parallel_per_cu_max > 0 && per_cu > parallel_per_cu_max) per_cu = parallel_per_cu_max;
    } else {
        // the column blocks of a wide X (grid.y) are resident side by side: count them in
        const long long want = (tiles * col_blocks + waves - 1) / waves;
        if (col_blocks > 1 && want <= blocks_per_cu) return clamp_blocks(cus * want / col_blocks, cap);
        per_cu = (tiles + waves - 1) / waves;
    }
    if (per_cu > blocks_per_cu) per_cu = blocks_per_cu;
    return (unsigned)(cus * per_cu);
}

// Which pipeline the balanced parallel kernel runs.  Blocks of entries with the next block's gathers in flight
// during the row logic (nb_pr_kernel) for up to four dense columns per lane on matrices of six million entries
// and more: 2-6 % faster there on R-MAT matrices of every skew (2^20 vertices, degree 16, power law: 104 -> 98 us
// per call at N = 1, main launch 98 -> 90 us; N = 3: 122 -> 116 us, N = 4: 125 -> 120 us) and on random columns; not
// on banded matrices (see launch_nb_pr_v).  Smaller matrices give a wave only a few blocks, and the longer kernel's
// start-up costs more than the overlap returns (5-10 % slower from 0.25 to 4 million entries), so they keep the
// tiles of merge-path items (nb_pr_tiled_kernel), as does a call that does not know its entry count.  With eight
// columns per lane the registers that hold a block's gathered values cost more occupancy than the overlap gives
// (R-MAT N = 8: 162 -> 178 us): tiles as well.  DGSP_ABL_ITEM_TILES / DGSP_ABL_ENTRY_BLOCKS force one or the other
// where both exist (the comparison for this choice).
template <int V>
constexpr bool kNbPrStreams = V <= 4;
constexpr long long kNbPrStreamNnzMin = 6000000;

template <int V, int KQ>
int launch_nb_pr_v(const Problem& p) {
    constexpr unsigned tile = kWave * 4 * KQ;
    const unsigned col_groups = (unsigned)((p.N + V - 1) / V);      // V = 8 also takes N = 5, 6, 7: one group
    // the row store addresses a step's rows with 32-bit byte offsets: tile rows * N * 4 must fit
    if (col_groups > 65535u || p.ldy > kBalancedLdyMax) return DGSP_ERR_UNSUPPORTED;
    const bool forced_blocks = (p.switches & (DGSP_ABL_ENTRY_BLOCKS | DGSP_ABL_SERIAL_SEGMENT_SCAN)) != 0;
    // A banded matrix (neighbouring rows share their columns: stencils, bands): its gathers hit the L1 and are bound
    // by the rate of the CU's address unit, not by latency, so gathers requested a block ahead gain nothing, and at up
    // to three columns per lane two workgroups per CU leave each wave more of the L1 than four do (27-point stencil on
    // 128^3 at N = 1: item tiles on 2 / 3 workgroups per CU 132 / 140 us, entry blocks on 2 / 3 / 4 155 / 139 / 143 us;
    // N = 2: 137 against 152 us; N = 3: 142 against 150 us; bands of 27 and 64: 116, 123 against 120, 134 us; with
    // four columns per lane the larger grid is as good: 153 / 148 / 149 us on 2 / 3 / 4).
    const bool banded_x = banded(p) && !forced_blocks;
    const bool tiled = !kNbPrStreams<V> || (p.switches & DGSP_ABL_ITEM_TILES) != 0 ||
                       (!forced_blocks && (p.nnz < kNbPrStreamNnzMin || banded_x));   // unknown entry count (-1): tiles
    int resident = resident_blocks_per_cu(nb_pr_tiled_kernel<V, KQ>);
    if constexpr (kNbPrStreams<V>) { if (!tiled) resident = resident_blocks_per_cu(nb_pr_kernel<V, KQ>); }
    const bool few_waves = banded_x && V <= 3;
    const dim3 grid(balanced_blocks(p, tile, resident, true, 1, few_waves ? 2 : 0), col_groups);
    if (p.phase != DGSP_PHASE_MAIN)
        if (int rc = launch_prepare(p, grid.x * kWavesPerBlock * kSubRanges, 6, -1)) return rc;
    if (p.phase != DGSP_PHASE_PREPARE) {
        if (tiled) {
            if (p.scaled)
                DGSP_LAUNCH((nb_pr_tiled_kernel<V, KQ, true>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X,
                            p.Y, Scaling{p.alpha, p.beta});
            else
                DGSP_LAUNCH((nb_pr_tiled_kernel<V, KQ>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X, p.Y);
        } else if constexpr (kNbPrStreams<V>) {
            if constexpr (V <= 2) {
                if (p.switches & DGSP_ABL_SERIAL_SEGMENT_SCAN) {
                    DGSP_LAUNCH((nb_pr_kernel<V, KQ, false, true>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X, p.Y);
                    return DGSP_OK;
                }
            }
            if (p.scaled)
                DGSP_LAUNCH((nb_pr_kernel<V, KQ, true>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X, p.Y,
                            Scaling{p.alpha, p.beta});
            else
                DGSP_LAUNCH((nb_pr_kernel<V, KQ>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X, p.Y);
        }
    }
    return DGSP_OK;
}

int launch_nb_pr(const Problem& p) {
    switch (nb_pr_lane_width(p.N, p.switches)) {
        case 8: return launch_nb_pr_v<8, 1>(p);
        case 4: return launch_nb_pr_v<4, kNbPrKq>(p);
        case 3: return launch_nb_pr_v<3, kNbPrKq>(p);
        case 2: return launch_nb_pr_v<2, kNbPrKq>(p);
        default: return launch_nb_pr_v<1, kNbPrKq>(p);
    }
}

template <int V, bool XBUF, int DEPTH, bool RAGGED>
int launch_nb_sr_v(const Problem& p) {
    // N a multiple of 64: column blocks of 64 dense columns (256 bytes of a row of X), several blocks over
    // the same chunks, one after the other in launch order.  The rows of X that many matrix rows share (hub
    // columns of a power-law graph) then compete for the L2 with a quarter-kilobyte each instead of N * 4
    // bytes; re-reading the 8 bytes of an entry per block costs 3 % of what the block gathers for it.
    SrColumns cols = sr_columns(p.N, V, p.N >= 128);
    // comparison: column blocks of 32 dense columns (one 128-byte line of a row of X per entry and block)
    if ((p.switches & DGSP_ABL_COLUMN_BLOCKS_32) && V == 4 && p.N % 32 == 0 && p.N >= 64)
        cols = SrColumns{3, 32, (unsigned)(p.N / 32)};
    // A matrix with fewer tiles than the machine has room for waves (two per SIMD) leaves CUs idle: a wave takes a
    // whole tile of 512 items whatever N is.  Narrower column blocks make more workgroups out of the same tiles
    // (65 536 rows of 4 entries at N = 32: 640 tiles on 1024 SIMDs; two blocks of 16 columns instead of one of 32).
    // Only where entries make up most of the items: every block walks the row ends again, and in a matrix of
    // mostly empty rows that walk is the work (262 144 rows with 52 000 entries at N = 32: 33 -> 56 us when split).
    if (p.nnz >= p.M) {
        const long long tiles = (p.nnz + (long long)p.M + kNbSrTile - 1) / kNbSrTile;
        const long long room = (long long)device_info().cus * kWavesPerBlock * 2;
        while (tiles * cols.blocks < room && cols.logG > 0 && cols.cols_per_block % (2 * V) == 0) {
            const int per = cols.cols_per_block / 2;
            cols = SrColumns{sr_lanes_log2(per, V), per, (unsigned)((p.N + per - 1) / per)};
        }
    }
    const int logG = cols.logG;
    const unsigned col_blocks = cols.blocks;
    if (col_blocks > 65535u) return DGSP_ERR_INVALID_ARG;
    const int logU = kNbSrLogTile - 6 + logG;   // items per lane-group run
    // a tile's rows are stored through 32-bit byte offsets from the tile's first row
    if (p.ldy > kBalancedLdyMax) return DGSP_ERR_UNSUPPORTED;
    dim3 grid(balanced_blocks(p, kNbSrTile, resident_blocks_per_cu(nb_sr_kernel<V, XBUF, DEPTH, false, RAGGED>), false, col_blocks), col_blocks);
    // Two or four column blocks of a wide X (N = 128 ... 256): every XCD works on one block only, so that an L2 sees
    // one block's slice of X and the slices do not compete (R-MAT 2^20 at N = 128: 1125 -> 1062 us, N = 256: 2154 ->
    // 2097 us; uniform columns: 0 ... +4 %).  With eight blocks (N = 512) every XCD would walk the whole matrix alone,
    // which measured 10-20 % slower on every matrix tried: from there on the blocks stay a second grid dimension.
    // The grid is then one-dimensional with whole workgroups per XCD.  DGSP_ABL_BLOCKS_OFF_XCDS keeps the blocks as
    // a second grid dimension (the comparison); eight blocks of 32 columns (DGSP_ABL_COLUMN_BLOCKS_32 at N = 256)
    // are tied to XCDs too, so that both comparisons can be combined.
    unsigned pinned = 0;
    if (!(p.switches & DGSP_ABL_BLOCKS_OFF_XCDS) && p.N >= 128 &&
        (col_blocks == 2 || col_blocks == 4 || (col_blocks == 8 && (p.switches & DGSP_ABL_COLUMN_BLOCKS_32)))) {
        pinned = col_blocks;
        const unsigned per_xcd = (grid.x * col_blocks + kXcd - 1) / kXcd;         // as many workgroups as before, in one dimension
        grid = dim3(per_xcd * kXcd, 1);
    }
    const unsigned chunk_groups = pinned ? grid.x / pinned : grid.x;              // workgroups that share one chunk list
    if (p.phase != DGSP_PHASE_MAIN)
        if (int rc = launch_prepare(p, chunk_groups * kWavesPerBlock * kSubRanges, (unsigned)logU, kNbSrLogTile)) return rc;
    if (p.phase != DGSP_PHASE_PREPARE) {
        if (p.scaled) {
            DGSP_LAUNCH((nb_sr_kernel<V, XBUF, DEPTH, true, RAGGED>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx,
                        p.vals, p.X, p.Y, logG, cols.cols_per_block, Scaling{p.alpha, p.beta}, pinned);
        } else {
            DGSP_LAUNCH((nb_sr_kernel<V, XBUF, DEPTH, false, RAGGED>), grid, p.M, p.K, p.N, p.ldx, p.ldy, p.rowptr, p.colidx, p.vals, p.X, p.Y,
                        logG, cols.cols_per_block, Scaling{1.0f, 0.0f}, pinned);
        }
    }
    return DGSP_OK;
}

template <int V, bool RAGGED>
int launch_nb_sr_pick(const Problem& p) {
    const bool xb = x_fits_descriptor(p);
    if (banded(p)) return xb ? launch_nb_sr_v<V, true, 4, RAGGED>(p) : launch_nb_sr_v<V, false, 4, RAGGED>(p);
    constexpr int D = sr_depth_scattered<V>();
    return xb ? launch_nb_sr_v<V, true, D, RAGGED>(p) : launch_nb_sr_v<V, false, D, RAGGED>(p);
}

int launch_nb_sr(const Problem& p) {
    const SrShape shape = sr_shape(p);
    switch (shape.v) {
        case 4: return shape.ragged ? launch_nb_sr_pick<4, true>(p) : launch_nb_sr_pick<4, false>(p);
        case 2: return launch_nb_sr_pick<2, false>(p);
        default: return launch_nb_sr_pick<1, false>(p);
    }
}

// ---------------------------------------------------------------- selector state
// Defaults fitted on MI355X on the 24-matrix synthetic sweep, pr_nnz_max on larger
// banded and random matrices (the paper prints no threshold values, Section 2.2).
std::mutex g_thresholds_mu;                 // guards g_thresholds: readers take a copy
dgsp_thresholds_t g_thresholds = {
    /* n_parallel_max  */ 4,
    /* pr_avg_row_min  */ 48.0,
    /* pr_cv_max       */ 0.05,
    /* sr_cv_min       */ 0.3,
    /* sr_stdv_min     */ 3.0,
    /* pr_nnz_max      */ 20000000,
    /* short_avg_row_max */ 20.0,
    /* short_max_row_max */ 64,
    /* wide_parallel_n   */ 8,
    /* big_x_bytes_min   */ 6000000,
    /* big_x_cv_max      */ 0.2,
    /* big_x_avg_row_max */ 64.0,
    /* short_min_waves   */ 2048,
    /* pr_small_nnz_max  */ 2000000,
    /* pr_small_cv_max   */ 0.6,
};

dgsp_thresholds_t thresholds_snapshot() {
    std::lock_guard<std::mutex> lock(g_thresholds_mu);
    return g_thresholds;
}

// The balanced kernels address the rows of a tile through 32-bit byte offsets and stop at a leading dimension
// of 2^20 floats (DGSP_ERR_UNSUPPORTED when asked for by name).  A choice the library makes itself moves to the
// row-split sequential kernel there, which has no such limit (so wide a Y means N or the stride is huge).
inline int library_choice(int algo, int64_t ldy) {
    return ((algo == DGSP_NB_SR || algo == DGSP_NB_PR) && ldy > kBalancedLdyMax) ? DGSP_RS_SR : algo;
}

int run(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr, const int32_t* colidx,
        const float* vals, const float* X, float* Y, int algo, void* stream, int phase = DGSP_PHASE_ALL,
        Hints hints = Hints(), int switches = 0, int64_t ldx = -1, int64_t ldy = -1, const Scaling* scaling = nullptr) {
    if (M < 0 || K < 0 || N < 0) return DGSP_ERR_INVALID_ARG;
    if (ldx < 0) ldx = N;            // packed rows unless the caller says otherwise
    if (ldy < 0) ldy = N;
    if (ldx < N || ldy < N) return DGSP_ERR_INVALID_ARG;
    if (algo < DGSP_AUTO || algo > DGSP_NB_PR) return DGSP_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return DGSP_OK;
    // int32 index range; a little headroom keeps position arithmetic simple
    const int64_t lim = (int64_t)INT32_MAX - 4096;
    if (M > lim || K > lim || N > lim || nnz > lim || ldx > lim || ldy > lim) return DGSP_ERR_INVALID_ARG;
    if (!rowptr || !Y) return DGSP_ERR_INVALID_ARG;
    if (nnz > 0 && (!colidx || !vals || !X || K == 0)) return DGSP_ERR_INVALID_ARG;

    // no row statistics: the balanced kernels are safe for any row-length distribution; the parallel one while
    // it needs a single pass over the matrix (it was the faster of the two on 22 of 24 sweep matrices at N = 8)
    if (algo == DGSP_AUTO) {
        const dgsp_thresholds_t t = thresholds_snapshot();
        const int64_t one_pass = t.wide_parallel_n > t.n_parallel_max ? t.wide_parallel_n : t.n_parallel_max;
        algo = library_choice((N <= one_pass) ? DGSP_NB_PR : DGSP_NB_SR, ldy);
    }

    Problem p{(int)M, (int)N, (int)ldx, (int)ldy, K, nnz, rowptr, colidx, vals, X, Y, (hipStream_t)stream, phase, hints.col_span, hints.cv_row, switches};
    if (scaling) { p.scaled = true; p.alpha = scaling->alpha; p.beta = scaling->beta; }
    switch (algo) {
        case DGSP_RS_SR: return phase == DGSP_PHASE_PREPARE ? DGSP_OK : launch_rs_sr(p);
        case DGSP_RS_PR: return phase == DGSP_PHASE_PREPARE ? DGSP_OK : launch_rs_pr(p);
        case DGSP_NB_SR: return launch_nb_sr(p);
        default: return launch_nb_pr(p);
    }
}

}  // namespace

// ==================================================================== C-ABI

extern "C" int dgsp_spmm_csr(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx,
                             const float* vals, const float* X, float* Y, int algo, void* stream) {
    return run(M, K, N, -1, rowptr, colidx, vals, X, Y, algo, stream);
}

extern "C" int dgsp_spmm_csr_nnz(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                                 const int32_t* colidx, const float* vals, const float* X, float* Y, int algo,
                                 void* stream) {
    return run(M, K, N, nnz < 0 ? -1 : nnz, rowptr, colidx, vals, X, Y, algo, stream);
}

extern "C" int dgsp_spmm_csr_phase(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                                   const int32_t* colidx, const float* vals, const float* X, float* Y, int algo,
                                   int phase, const dgsp_features_t* features, void* stream) {
    if (algo < DGSP_RS_SR || algo > DGSP_NB_PR) return DGSP_ERR_INVALID_ARG;
    if (phase < DGSP_PHASE_ALL || phase > DGSP_PHASE_MAIN) return DGSP_ERR_INVALID_ARG;
    if (features && nnz < 0) nnz = features->nnz;
    return run(M, K, N, nnz < 0 ? -1 : nnz, rowptr, colidx, vals, X, Y, algo, stream, phase,
               Hints(features));
}

extern "C" int dgsp_spmm_csr_ld(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                                const int32_t* colidx, const float* vals, const float* X, int64_t ldx, float* Y,
                                int64_t ldy, int algo, const dgsp_features_t* features, void* stream) {
    if (ldx < N || ldy < N) return DGSP_ERR_INVALID_ARG;
    if (features && nnz < 0) nnz = features->nnz;
    if (algo == DGSP_AUTO && features && N >= 1) {
        algo = library_choice(dgsp_select_algo(features, N), ldy);
    }
    return run(M, K, N, nnz < 0 ? -1 : nnz, rowptr, colidx, vals, X, Y, algo, stream, DGSP_PHASE_ALL,
               Hints(features), 0, ldx, ldy);
}

extern "C" int dgsp_spmm_csr_axpby(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                                   const int32_t* colidx, const float* vals, const float* X, int64_t ldx, float* Y,
                                   int64_t ldy, float alpha, float beta, int algo, const dgsp_features_t* features,
                                   void* stream) {
    if (ldx < N || ldy < N) return DGSP_ERR_INVALID_ARG;
    if (features && nnz < 0) nnz = features->nnz;
    if (algo == DGSP_AUTO && features && N >= 1) {
        algo = library_choice(dgsp_select_algo(features, N), ldy);
    }
    const Scaling sc{alpha, beta};
    return run(M, K, N, nnz < 0 ? -1 : nnz, rowptr, colidx, vals, X, Y, algo, stream, DGSP_PHASE_ALL,
               Hints(features), 0, ldx, ldy, &sc);
}

extern "C" int dgsp_spmm_csr_ablation(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                                      const int32_t* colidx, const float* vals, const float* X, float* Y, int algo,
                                      int switches, const dgsp_features_t* features, void* stream) {
    if (algo < DGSP_RS_SR || algo > DGSP_NB_PR) return DGSP_ERR_INVALID_ARG;
    if (switches & ~(DGSP_ABL_SCALAR_DENSE_LOADS | DGSP_ABL_NO_SPARSE_STAGING | DGSP_ABL_ITEM_TILES | DGSP_ABL_SERIAL_SEGMENT_SCAN |
                     DGSP_ABL_COLUMN_BLOCKS_32 | DGSP_ABL_BLOCKS_OFF_XCDS | DGSP_ABL_ENTRY_BLOCKS))
        return DGSP_ERR_INVALID_ARG;
    if ((switches & DGSP_ABL_ENTRY_BLOCKS) &&
        (algo != DGSP_NB_PR || (switches & DGSP_ABL_ITEM_TILES) || nb_pr_lane_width(N, switches) > 4))
        return DGSP_ERR_UNSUPPORTED;
    if ((switches & (DGSP_ABL_COLUMN_BLOCKS_32 | DGSP_ABL_BLOCKS_OFF_XCDS)) && algo != DGSP_NB_SR) return DGSP_ERR_UNSUPPORTED;
    if ((switches & DGSP_ABL_NO_SPARSE_STAGING) && algo != DGSP_RS_SR) return DGSP_ERR_UNSUPPORTED;
    if ((switches & DGSP_ABL_ITEM_TILES) && algo != DGSP_NB_PR) return DGSP_ERR_UNSUPPORTED;
    if (switches & DGSP_ABL_SERIAL_SEGMENT_SCAN) {
        // offered at one or two dense columns per lane (on the entry-block pipeline)
        const bool narrow = nb_pr_lane_width(N, switches) <= 2;
        if (algo != DGSP_NB_PR || (switches & DGSP_ABL_ITEM_TILES) || !narrow) return DGSP_ERR_UNSUPPORTED;
    }
    if (features && nnz < 0) nnz = features->nnz;
    return run(M, K, N, nnz < 0 ? -1 : nnz, rowptr, colidx, vals, X, Y, algo, stream, DGSP_PHASE_ALL,
               Hints(features), switches);
}

extern "C" int dgsp_spmm_csr_auto(int64_t M, int64_t K, int64_t N, const dgsp_features_t* features,
                                  const int32_t* rowptr, const int32_t* colidx, const float* vals, const float* X,
                                  float* Y, int* chosen, void* stream) {
    if (!features) return DGSP_ERR_INVALID_ARG;
    if (features->M != M || features->nnz < 0) return DGSP_ERR_INVALID_ARG;
    int algo = (N >= 1) ? library_choice(dgsp_select_algo(features, N), N) : DGSP_NB_PR;
    if (algo < 0) return DGSP_ERR_INVALID_ARG;
    if (chosen) *chosen = algo;
    return run(M, K, N, features->nnz, rowptr, colidx, vals, X, Y, algo, stream, DGSP_PHASE_ALL, Hints(features));
}

// ---------------------------------------------------------------- 64-bit row pointers
namespace {
constexpr int64_t kSlabEntries = 1ll << 30;        // a slab holds this many entries plus at most one row more
inline int64_t slab_count(int64_t nnz) { return nnz <= 0 ? 1 : (nnz + kSlabEntries - 1) / kSlabEntries; }
inline int64_t round_up16(int64_t v) { return (v + 15) / 16 * 16; }
}  // namespace

extern "C" int64_t dgsp_spmm_csr_i64_workspace_bytes(int64_t M, int64_t nnz) {
    if (M < 0 || nnz < 0) return -1;
    return round_up16(4 * (M + 1)) + 16 * (slab_count(nnz) + 1);
}

extern "C" int dgsp_spmm_csr_i64(int64_t M, int64_t K, int64_t N, int64_t nnz, const int64_t* rowptr, const int32_t* colidx,
                                 const float* vals, const float* X, float* Y, int algo, void* workspace,
                                 int64_t workspace_bytes, void* stream) {
    if (M < 0 || K < 0 || N < 0 || nnz < 0) return DGSP_ERR_INVALID_ARG;
    if (algo < DGSP_AUTO || algo > DGSP_NB_PR) return DGSP_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return DGSP_OK;
    const int64_t lim = (int64_t)INT32_MAX - 4096;
    if (M > lim || K > lim || N > lim) return DGSP_ERR_INVALID_ARG;
    if (!rowptr || !Y || (nnz > 0 && (!colidx || !vals || !X || K == 0))) return DGSP_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 16) || workspace_bytes < dgsp_spmm_csr_i64_workspace_bytes(M, nnz))
        return DGSP_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int nslabs = (int)slab_count(nnz);
    int* rowptr32 = static_cast<int*>(workspace);
    long long* cuts = reinterpret_cast<long long*>(static_cast<char*>(workspace) + round_up16(4 * (M + 1)));
    hipLaunchKernelGGL(i64_slab_bounds_kernel, dim3((unsigned)((nslabs + 1 + kWave - 1) / kWave)), dim3(kWave), 0, st,
                       (long long)M, reinterpret_cast<const long long*>(rowptr), nslabs, (long long)kSlabEntries, cuts);
    if (hipGetLastError() != hipSuccess) return DGSP_ERR_LAUNCH;
    // the cuts decide launch sizes, so the host has to see them: the one wait of this entry point
    long long h[2 * 16];
    if (nslabs + 1 > 16) return DGSP_ERR_UNSUPPORTED;                   // 15 * 2^30 entries and more
    if (hipMemcpyAsync(h, cuts, sizeof(long long) * 2 * (size_t)(nslabs + 1), hipMemcpyDeviceToHost, st) != hipSuccess)
        return DGSP_ERR_LAUNCH;
    if (hipStreamSynchronize(st) != hipSuccess) return DGSP_ERR_LAUNCH;
    if (h[1] != 0 || h[2 * nslabs + 1] != nnz) return DGSP_ERR_INVALID_ARG;      // rowptr[0] != 0 or rowptr[M] != nnz
    for (int k = 0; k < nslabs; ++k)
        if (h[2 * k + 3] - h[2 * k + 1] > lim || h[2 * k + 3] < h[2 * k + 1] || h[2 * k + 2] < h[2 * k]) return DGSP_ERR_UNSUPPORTED;
    for (int k = 0; k < nslabs; ++k) {
        const int64_t first = h[2 * k], rows = h[2 * k + 2] - first;
        const int64_t base = h[2 * k + 1], entries = h[2 * k + 3] - base;
        if (rows == 0) continue;
        const long long cap = (long long)device_info().cus * kBlocksPerCu * 4;
        hipLaunchKernelGGL(i64_slab_rowptr_kernel, dim3(clamp_blocks((rows + 1 + kBlock - 1) / kBlock, cap)), dim3(kBlock), 0, st,
                           (long long)rows, reinterpret_cast<const long long*>(rowptr) + first, (long long)base, rowptr32);
        if (hipGetLastError() != hipSuccess) return DGSP_ERR_LAUNCH;
        const int rc = run(rows, K, N, entries, rowptr32, colidx ? colidx + base : nullptr, vals ? vals + base : nullptr, X,
                           Y + (size_t)first * (size_t)N, algo, stream);
        if (rc != DGSP_OK) return rc;
    }
    return DGSP_OK;
}

// Section 2.2: N picks the reduction, row-length statistics pick the partition.
extern "C" int dgsp_select_algo(const dgsp_features_t* f, int64_t N) {
    if (!f || N < 1) return DGSP_AUTO;
    const dgsp_thresholds_t t = thresholds_snapshot();
    // all rows short: one lane group per row keeps a wave busy with no cross-lane step and no idle tail - provided
    // the rows fill the machine: the row-split sequential kernel runs M * (lanes per row) / 64 waves
    if (f->nnz > 0 && f->avg_row <= t.short_avg_row_max && f->max_row <= t.short_max_row_max) {
        const int lanes_log2 = N < 4 ? 0 : sr_lanes_log2(N, 4);
        if ((double)f->M * (double)(1 << lanes_log2) >= 64.0 * (double)t.short_min_waves) return DGSP_RS_SR;
    }
    if (N <= t.n_parallel_max) {
        // X beyond one L2, rows alike and spread over all columns: one row per lane sweeps X in step
        if (t.big_x_bytes_min > 0 && (double)f->K * (double)N * 4.0 >= (double)t.big_x_bytes_min &&
            f->cv_row <= t.big_x_cv_max && f->avg_row <= t.big_x_avg_row_max && f->col_span >= 0.5)
            return DGSP_RS_SR;
        // a small matrix of about equal rows: the balanced kernel's second launch (4-6 us) is a third of the call
        if (f->nnz > 0 && f->nnz <= t.pr_small_nnz_max && f->cv_row <= t.pr_small_cv_max) return DGSP_RS_PR;
        // parallel reduction: long rows keep a row's lanes busy, short rows idle them
        const bool row_split = f->avg_row >= t.pr_avg_row_min && f->cv_row <= t.pr_cv_max && f->nnz < t.pr_nnz_max;
        return row_split ? DGSP_RS_PR : DGSP_NB_PR;
    }
    // sequential reduction: balance only when stdv_row / avg_row says rows are uneven
    if (!(f->cv_row > t.sr_cv_min && f->stdv_row > t.sr_stdv_min)) return DGSP_RS_SR;
    // up to eight columns fit one lane of the balanced parallel kernel: still a single pass
    return (N <= t.wide_parallel_n) ? DGSP_NB_PR : DGSP_NB_SR;
}

extern "C" void dgsp_get_thresholds(dgsp_thresholds_t* out) {
    if (out) *out = thresholds_snapshot();
}

extern "C" void dgsp_set_thresholds(const dgsp_thresholds_t* in) {
    if (!in) return;
    std::lock_guard<std::mutex> lock(g_thresholds_mu);
    g_thresholds = *in;
}

extern "C" int dgsp_features_from_rowptr_host(int64_t M, int64_t K, const int32_t* rowptr, dgsp_features_t* out) {
    if (M < 0 || K < 0 || !out || (!rowptr && M > 0)) return DGSP_ERR_INVALID_ARG;
    dgsp_features_t f{};
    f.M = M; f.K = K;
    if (M == 0) { *out = f; return DGSP_OK; }
    if (rowptr[0] != 0) return DGSP_ERR_INVALID_ARG;
    // one pass: sum and sum of squares in integers (exact), min and max
    unsigned __int128 sq = 0;
    int64_t mx = 0, mn = INT64_MAX;
    for (int64_t i = 0; i < M; ++i) {
        const int64_t len = (int64_t)rowptr[i + 1] - (int64_t)rowptr[i];
        if (len < 0) return DGSP_ERR_INVALID_ARG;
        sq += (unsigned __int128)((uint64_t)len * (uint64_t)len);
        mx = len > mx ? len : mx;
        mn = len < mn ? len : mn;
    }
    f.nnz = rowptr[M];
    f.max_row = mx; f.min_row = mn;
    f.avg_row = (double)f.nnz / (double)M;
    // population variance = E[len^2] - avg^2, formed from exact integers:
    // (M * sum len^2 - nnz^2) / M^2
    const unsigned __int128 num = sq * (unsigned __int128)M - (unsigned __int128)((uint64_t)f.nnz) * (uint64_t)f.nnz;
    const double var = (double)num / ((double)M * (double)M);
    f.stdv_row = std::sqrt(var);
    f.cv_row = f.avg_row > 0 ? f.stdv_row / f.avg_row : 0.0;
    f.col_span = 0.0;
    *out = f;
    return DGSP_OK;
}

constexpr int kGatherProbeBlocks = 4096;

extern "C" int64_t dgsp_gather_probe_out_len(void) { return (int64_t)kGatherProbeBlocks * kBlock; }

extern "C" int dgsp_gather_probe(float* out, const float* x, const int32_t* idx, int64_t n, void* stream) {
    if (n < 0 || !out || (n > 0 && (!x || !idx))) return DGSP_ERR_INVALID_ARG;
    hipLaunchKernelGGL(gather_probe_kernel, dim3(kGatherProbeBlocks), dim3(kBlock), 0, (hipStream_t)stream, out, x,
                       idx, (long long)n);
    return hipGetLastError() == hipSuccess ? DGSP_OK : DGSP_ERR_LAUNCH;
}

// ---------------------------------------------------------------- floor probes (measurement aids)
namespace {
// four workgroups per CU: what the lean pipeline ran best with (512 / 1024 / 1280 / 2048 workgroups on the R-MAT
// SpMV: 79 / 82 / 90 / 86 us; on the stencil: 118 / 110 / 152 / 114 us)
constexpr int kStreamProbeBlocks = 1024;

struct RowProbeShape { int logG; unsigned col_blocks; unsigned blocks; };
RowProbeShape row_probe_shape(int64_t N) {
    const int logG = sr_lanes_log2(N, 4, 4);                               // at most 16 lanes = 64 columns per group
    const unsigned col_blocks = (unsigned)((N + (4 << logG) - 1) / (4 << logG));
    const unsigned blocks = (unsigned)(device_info().cus * resident_blocks_per_cu(row_gather_probe_kernel));
    return {logG, col_blocks, blocks};
}
}  // namespace

extern "C" int64_t dgsp_floor_probe_out_len(int mode, int64_t N) {
    if (mode == DGSP_PROBE_GATHER) return dgsp_gather_probe_out_len();
    if (mode == DGSP_PROBE_STREAM_GATHER_FMA) return (N == 1 || N == 2 || N == 4) ? (int64_t)kStreamProbeBlocks * kBlock * N : -1;
    if (mode == DGSP_PROBE_ROW_GATHER) {
        if (N < 4 || N % 4 != 0) return -1;
        const RowProbeShape sh = row_probe_shape(N);
        return (int64_t)sh.blocks * sh.col_blocks * kBlock * 4;
    }
    return -1;
}

extern "C" int dgsp_floor_probe(int mode, int64_t nnz, int64_t K, int64_t N, const int32_t* colidx, const float* vals,
                                const float* X, float* out, void* stream) {
    if (nnz < 0 || K < 1 || N < 1 || !out || !X || (nnz > 0 && !colidx)) return DGSP_ERR_INVALID_ARG;
    const int64_t lim = (int64_t)INT32_MAX - 4096;
    if (nnz > lim || K > lim || N > (1 << 20)) return DGSP_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (mode == DGSP_PROBE_GATHER) {
        if (N != 1) return DGSP_ERR_UNSUPPORTED;
        return dgsp_gather_probe(out, X, colidx, nnz, stream);
    }
    if (nnz > 0 && !vals) return DGSP_ERR_INVALID_ARG;
    if (mode == DGSP_PROBE_STREAM_GATHER_FMA) {
        const dim3 grid(kStreamProbeBlocks);
        switch (N) {
            case 1: hipLaunchKernelGGL(stream_gather_fma_probe_kernel<1>, grid, dim3(kBlock), 0, st, out, X, (long long)K, 1, colidx, vals, (long long)nnz); break;
            case 2: hipLaunchKernelGGL(stream_gather_fma_probe_kernel<2>, grid, dim3(kBlock), 0, st, out, X, (long long)K, 2, colidx, vals, (long long)nnz); break;
            case 4: hipLaunchKernelGGL(stream_gather_fma_probe_kernel<4>, grid, dim3(kBlock), 0, st, out, X, (long long)K, 4, colidx, vals, (long long)nnz); break;
            default: return DGSP_ERR_UNSUPPORTED;
        }
        return hipGetLastError() == hipSuccess ? DGSP_OK : DGSP_ERR_LAUNCH;
    }
    if (mode == DGSP_PROBE_ROW_GATHER) {
        if (N < 4 || N % 4 != 0) return DGSP_ERR_UNSUPPORTED;
        const RowProbeShape sh = row_probe_shape(N);
        if (sh.col_blocks > 65535u) return DGSP_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(row_gather_probe_kernel, dim3(sh.blocks, sh.col_blocks), dim3(kBlock), 0, st, out, X, (long long)K,
                           (int)N, (int)N, colidx, vals, (long long)nnz, sh.logG);
        return hipGetLastError() == hipSuccess ? DGSP_OK : DGSP_ERR_LAUNCH;
    }
    return DGSP_ERR_INVALID_ARG;
}

extern "C" int dgsp_features_from_csr_host(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colidx,
                                           dgsp_features_t* out) {
    const int rc = dgsp_features_from_rowptr_host(M, K, rowptr, out);
    if (rc != DGSP_OK) return rc;
    if (out->nnz > 0 && !colidx) return DGSP_ERR_INVALID_ARG;
    if (M == 0 || K == 0 || out->nnz == 0) return DGSP_OK;
    // mean over the non-empty rows of (largest - smallest column + 1) / K; the spans are summed as
    // integers so that the device version, which adds them in any order, gives the same bits
    uint64_t sum = 0;
    int64_t rows = 0;
    for (int64_t i = 0; i < M; ++i) {
        const int64_t s = rowptr[i], e = rowptr[i + 1];
        if (s == e) continue;
        int32_t lo = colidx[s], hi = colidx[s];
        if (colidx[e - 1] < lo || e - s <= 2) {
            for (int64_t p = s; p < e; ++p) { lo = colidx[p] < lo ? colidx[p] : lo; hi = colidx[p] > hi ? colidx[p] : hi; }
        } else {
            // sorted rows (the usual case) need only their two ends; verify cheaply, else scan
            bool sorted = true;
            for (int64_t p = s + 1; p < e; ++p) if (colidx[p] < colidx[p - 1]) { sorted = false; break; }
            if (sorted) hi = colidx[e - 1];
            else for (int64_t p = s; p < e; ++p) { lo = colidx[p] < lo ? colidx[p] : lo; hi = colidx[p] > hi ? colidx[p] : hi; }
        }
        sum += (uint64_t)((int64_t)hi - (int64_t)lo + 1);
        ++rows;
    }
    out->col_span = rows ? (double)sum / ((double)K * (double)rows) : 0.0;
    return DGSP_OK;
}

namespace {

// The device pass behind both entry points: `ws` is kFeatureWords 64-bit words of device scratch.
int features_from_csr_device(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colidx,
                             unsigned long long* ws, dgsp_features_t* out, hipStream_t st) {
    dgsp_features_t f{};
    f.M = M; f.K = K;
    hipLaunchKernelGGL(features_init_kernel, dim3(1), dim3(kWave), 0, st, ws);
    const long long waves = (M + kWave - 1) / kWave;
    const dim3 grid(clamp_blocks((waves + kWavesPerBlock - 1) / kWavesPerBlock, (long long)device_info().cus * kBlocksPerCu));
    hipLaunchKernelGGL(features_kernel, grid, dim3(kBlock), 0, st, (int)M, rowptr, K > 0 ? colidx : nullptr, ws);
    if (hipGetLastError() != hipSuccess) return DGSP_ERR_LAUNCH;
    unsigned long long h[kFeatureWords];
    if (hipMemcpyAsync(h, ws, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess) return DGSP_ERR_LAUNCH;
    if (hipStreamSynchronize(st) != hipSuccess) return DGSP_ERR_LAUNCH;
    if (h[5] != 0 || h[6] != 0) return DGSP_ERR_INVALID_ARG;       // decreasing row pointers, rowptr[0] != 0
    f.nnz = (int64_t)h[7];
    f.max_row = (int64_t)h[1]; f.min_row = (int64_t)h[2];
    f.avg_row = (double)f.nnz / (double)M;
    const unsigned __int128 num = (unsigned __int128)h[0] * (unsigned __int128)M
                                  - (unsigned __int128)((uint64_t)f.nnz) * (uint64_t)f.nnz;
    f.stdv_row = std::sqrt((double)num / ((double)M * (double)M));
    f.cv_row = f.avg_row > 0 ? f.stdv_row / f.avg_row : 0.0;
    f.col_span = (colidx && K > 0 && h[3] > 0) ? (double)h[4] / ((double)K * (double)h[3]) : 0.0;
    *out = f;
    return DGSP_OK;
}

}  // namespace

extern "C" int dgsp_features_from_csr_device(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colidx,
                                             void* workspace, dgsp_features_t* out, void* stream) {
    if (M < 0 || K < 0 || !out || (!rowptr && M > 0)) return DGSP_ERR_INVALID_ARG;
    if (M > (int64_t)INT32_MAX - 4096) return DGSP_ERR_INVALID_ARG;
    if (M == 0) { dgsp_features_t f{}; f.K = K; *out = f; return DGSP_OK; }
    if (!workspace || !aligned(workspace, 8)) return DGSP_ERR_INVALID_ARG;
    return features_from_csr_device(M, K, rowptr, colidx, static_cast<unsigned long long*>(workspace), out,
                                    (hipStream_t)stream);
}

// ---------------------------------------------------------------- the entry point that allocates nothing
// The statistics pass with its scratch words in a static device array.  In host code the array's name is only
// a handle: the address a kernel can use comes from hipGetSymbolAddress, asked once per device with that
// device current (every GPU holds its own copy of the array at its own address).
static __device__ __align__(256) unsigned long long scratch[dgsp::kFeatureWords];     // 64 bytes per GPU

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned long long* g_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of `scratch` (nullptr on failure).
unsigned long long* scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = static_cast<unsigned long long*>(ptr);
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int dgsp_features_from_csr_device_noalloc(int64_t M, int64_t K, const int32_t* rowptr,
                                                     const int32_t* colidx, dgsp_features_t* out, void* stream) {
    if (M < 0 || K < 0 || !out || (!rowptr && M > 0)) return DGSP_ERR_INVALID_ARG;
    if (M > DGSP_FEATURES_NOALLOC_MAX_ROWS) return DGSP_ERR_INVALID_ARG;
    if (M == 0) { dgsp_features_t f{}; f.K = K; *out = f; return DGSP_OK; }
    unsigned long long* ws = scratch_of_current_device();
    if (!ws) return DGSP_ERR_LAUNCH;
    // features_init_kernel (a kernel, not a memset) clears the array first: it keeps the last call's contents
    return features_from_csr_device(M, K, rowptr, colidx, ws, out, (hipStream_t)stream);
}

extern "C" int dgsp_autotune(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                             const int32_t* colidx, const float* vals, const float* X, float* Y,
                             const dgsp_features_t* features, int reps, float* ms, int* best, void* stream) {
    if (!best) return DGSP_ERR_INVALID_ARG;
    if (reps < 1) reps = 1;
    if (reps > 100) reps = 100;
    if (features && nnz < 0) nnz = features->nnz;
    const Hints hints(features);
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return DGSP_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return DGSP_ERR_LAUNCH; }
    float t[4];
    int rc = DGSP_OK;
    float best_ms = INFINITY;
    int best_algo = -1;
    for (int algo = DGSP_RS_SR; algo <= DGSP_NB_PR && rc == DGSP_OK; ++algo) {
        t[algo] = INFINITY;
        // one untimed call first (first-use costs, caches), then `reps` timed ones; keep the fastest
        for (int r = 0; r <= reps; ++r) {
            if (r > 0 && hipEventRecord(e0, st) != hipSuccess) { rc = DGSP_ERR_LAUNCH; break; }
            const int one = run(M, K, N, nnz < 0 ? -1 : nnz, rowptr, colidx, vals, X, Y, algo, stream, DGSP_PHASE_ALL,
                                hints);
            if (one == DGSP_ERR_UNSUPPORTED) break;            // this kernel does not take the shape: skip it
            if (one != DGSP_OK) { rc = one; break; }
            if (r == 0) continue;
            float dt = 0.0f;
            if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&dt, e0, e1) != hipSuccess) { rc = DGSP_ERR_LAUNCH; break; }
            t[algo] = dt < t[algo] ? dt : t[algo];
            if (dt > 20.0f * best_ms) break;                   // hopeless: do not repeat a kernel 20x off the pace
        }
        if (t[algo] < best_ms) { best_ms = t[algo]; best_algo = algo; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != DGSP_OK) return rc;
    if (hipStreamSynchronize(st) != hipSuccess) return DGSP_ERR_LAUNCH;
    if (ms) for (int a = 0; a < 4; ++a) ms[a] = t[a];
    if (best_algo < 0) {
        // nothing was timed (M == 0 or N == 0: every call returns at once): any kernel will do
        best_algo = (N <= thresholds_snapshot().n_parallel_max) ? DGSP_NB_PR : DGSP_NB_SR;
    }
    *best = best_algo;
    return DGSP_OK;
}

extern "C" int dgsp_copy_f32(float* dst, const float* src, int64_t n, void* stream) {
    if (n < 0 || (n > 0 && (!dst || !src))) return DGSP_ERR_INVALID_ARG;
    if (n == 0) return DGSP_OK;
    if (!aligned(dst, 16) || !aligned(src, 16)) return DGSP_ERR_INVALID_ARG;
    const long long cap = (long long)device_info().cus * kBlocksPerCu * 4;
    const dim3 grid(clamp_blocks((n / 4 + kBlock - 1) / kBlock, cap));
    hipLaunchKernelGGL(copy_kernel, grid, dim3(kBlock), 0, (hipStream_t)stream, dst, src, (long long)n);
    return hipGetLastError() == hipSuccess ? DGSP_OK : DGSP_ERR_LAUNCH;
}

extern "C" const char* dgsp_algo_name(int algo) {
    switch (algo) {
        case DGSP_RS_SR: return "rs_sr";
        case DGSP_RS_PR: return "rs_pr";
        case DGSP_NB_SR: return "nb_sr";
        case DGSP_NB_PR: return "nb_pr";
        case DGSP_AUTO: return "auto";
        default: return "unknown";
    }
}

extern "C" const char* dgsp_status_string(int status) {
    switch (status) {
        case DGSP_OK: return "ok";
        case DGSP_ERR_INVALID_ARG: return "invalid argument";
        case DGSP_ERR_UNSUPPORTED: return "unsupported";
        case DGSP_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}
