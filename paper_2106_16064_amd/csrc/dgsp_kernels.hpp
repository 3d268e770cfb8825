// The four CSR SpMV/SpMM kernels of the paper's design space (Section 2.1):
// {row-split, nnz-balanced} x {sequential, parallel reduction}, for gfx950.
//
// Common shape of all four
//   * 256-thread workgroups = 4 waves; every cooperative step is wave-local
//     (DPP moves or wave-private LDS), so there is no s_barrier anywhere.
//   * `V` is the vector width of dense-row accesses: one dword / dwordx2 /
//     dwordx3 / dwordx4 per lane, or two dwordx4 for V = 8 (vector-type
//     dense-row loading, Section 2.1.2).  The memory pipeline takes these at
//     any dword address, so the choice of V depends on N only, never on the
//     alignment of X and Y or on their leading dimensions.
//   * X and Y are row-major with leading dimensions ldx, ldy (floats per row,
//     >= N); only the N used columns of a row are touched.
//   * Grids are sized to the machine, not to the matrix: a wave walks a list
//     of row groups (row-split) or tiles (balanced).  That is what allows the
//     number of stored entries to be read on the device from rowptr[M].
#pragma once

#include "dgsp_device.hpp"

namespace dgsp {

// ===========================================================================
// Row-split, parallel reduction  (CSR-Vector lineage; Section 1, Fig. 2(c,d))
// ===========================================================================
//
// 2^logG lanes own a row: they load consecutive (colidx, val) pairs, each
// lane gathers V dense values with one vector load, multiplies, keeps V
// private partial sums, and the group is folded with the DPP scan (a plain
// merge tree is the special case of the segmented scan with fixed-width
// segments).  logG < 0 asks the kernel to derive it from rowptr[M] / M.
// A wave keeps kRsPrUnroll row groups in flight.  For N > V the columns are
// processed V at a time.

__host__ __device__ __forceinline__ int pr_lanes_log2(long long nnz, long long M) {
    // lanes per row ~ average row length, rounded up to a power of two in [2, 64]
    const double avg = M > 0 ? (double)nnz / (double)M : 0.0;
    int lg = 1;
    while (lg < 6 && (double)(1 << lg) < avg) ++lg;
    return lg;
}

constexpr int kRsPrUnroll = 4;   // row groups a wave keeps in flight

template <int V, bool XBUF, bool AXPBY = false>
__global__ __launch_bounds__(kBlock) void rs_pr_kernel(int M, long long K, int N, int ldx, int ldy, const int* __restrict__ rowptr,
                                                        const int* __restrict__ colidx,
                                                        const float* __restrict__ vals,
                                                        const float* __restrict__ X, float* __restrict__ Y,
                                                        int logG_in, Scaling sc = Scaling{1.0f, 0.0f}) {
    constexpr int U = kRsPrUnroll;
    const int lane = lane_id();
    const unsigned nnz = (unsigned)rowptr[M];
    const int logG = logG_in >= 0 ? logG_in : pr_lanes_log2(nnz, M);
    const int G = 1 << logG;
    const int gl = lane & (G - 1);              // lane inside the group
    const int g = lane >> logG;                 // group inside the wave
    const int rows_per_wave = kWave >> logG;    // at most 32: a row has at least two lanes
    const unsigned nwaves = gridDim.x * kWavesPerBlock;
    const unsigned gw = xcd_contiguous(blockIdx.x, gridDim.x) * kWavesPerBlock + wave_in_block();
    // a wave step covers U * rows_per_wave consecutive rows: U independent load -> gather -> reduce chains
    const unsigned rows_per_step = (unsigned)(U * rows_per_wave);
    const unsigned nsteps = ((unsigned)M + rows_per_step - 1) / rows_per_step;
    // XBUF: the dense operand is read through a descriptor (its byte offsets fit 32 bits)
    const __amdgpu_buffer_rsrc_t rx = make_buffer(X, XBUF ? dense_bytes(K, ldx, N) : 0ull);

    auto fetch_dense = [&](unsigned c, bool ok, int n0, float (&x)[V]) {
        if constexpr (XBUF) {
            buffer_load_vec<V>(rx, ok ? c * (unsigned)ldx * 4u + (unsigned)n0 * 4u : kOutOfRange, x);
        } else {
            load_vec_dword_aligned<V>(X + (size_t)c * ldx + n0, x);                      // c is 0 when switched off: a valid row
#pragma unroll
            for (int i = 0; i < V; ++i) x[i] = ok ? x[i] : 0.0f;
        }
    };

    for (int n0 = 0; n0 < N; n0 += V) {
        for (unsigned st = gw; st < nsteps; st += nwaves) {
            // Row bounds: lanes 0..rows_per_wave fetch consecutive rowptr entries with one coalesced
            // load per row group and every lane picks its row's pair from them (cross-lane read).
            // Letting all lanes of a group load the same two words costs the memory pipeline a
            // cycle per lane, as much as the gather itself.
            unsigned rs[U], re[U];
            const unsigned long long row0 = (unsigned long long)st * rows_per_step;
            const __amdgpu_buffer_rsrc_t rp = make_buffer(rowptr + row0, ((unsigned long long)M + 1 - row0) * 4ull);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const unsigned idx = (unsigned)(u * rows_per_wave + lane);
                const unsigned v = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(
                    rp, lane <= rows_per_wave ? idx * 4u : kOutOfRange, 0, 0);     // past rowptr[M]: 0
                rs[u] = (unsigned)__shfl((int)v, g);
                re[u] = (unsigned)__shfl((int)v, g + 1);
                if (row0 + (unsigned)(u * rows_per_wave + g) >= (unsigned long long)M) re[u] = rs[u];   // no such row
            }
            // the step's entries start at its first row's start: offsets from there stay small
            const unsigned base = (unsigned)uniform((int)rs[0]);
            const unsigned long long bytes = (unsigned long long)(nnz - (base < nnz ? base : nnz)) * 4ull;
            const __amdgpu_buffer_rsrc_t rc = make_buffer(colidx + base, bytes);
            const __amdgpu_buffer_rsrc_t ra = make_buffer(vals + base, bytes);
            // column and value of the entry at position p (zeros when switched off)
            auto fetch_entry = [&](unsigned p, bool ok, unsigned& c, float& a) {
                const unsigned off = ok ? (p - base) * 4u : kOutOfRange;
                c = (unsigned)buffer_stream_i32(rc, off);
                a = buffer_stream_f32(ra, off);
            };
            float acc[U][V];
            // first entry of every lane: for rows no longer than the group this is all there is
            {
                unsigned c[U]; float a[U], x[U][V];
#pragma unroll
                for (int u = 0; u < U; ++u) fetch_entry(rs[u] + gl, rs[u] + gl < re[u], c[u], a[u]);
#pragma unroll
                for (int u = 0; u < U; ++u) fetch_dense(c[u], rs[u] + gl < re[u], n0, x[u]);
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int i = 0; i < V; ++i) acc[u][i] = a[u] * x[u][i];
            }
            // the rest of longer rows, two gathers in flight per lane
#pragma unroll
            for (int u = 0; u < U; ++u) {
                for (unsigned p = rs[u] + gl + G; p < re[u]; p += 2u * G) {
                    unsigned c0, c1; float a0, a1, x0[V], x1[V];
                    const bool ok1 = p + G < re[u];
                    fetch_entry(p, true, c0, a0);
                    fetch_entry(p + G, ok1, c1, a1);
                    fetch_dense(c0, true, n0, x0);
                    fetch_dense(c1, ok1, n0, x1);
#pragma unroll
                    for (int i = 0; i < V; ++i) acc[u][i] = fmaf(a1, x1[i], fmaf(a0, x0[i], acc[u][i]));
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                segmented_scan<V>(acc[u], gl, lane, G);   // all 64 lanes arrive here together
                const unsigned long long row = row0 + (unsigned)(u * rows_per_wave + g);
                if (row < (unsigned long long)M && gl == G - 1) {
                    float* y = Y + (size_t)row * ldy + n0;
                    if constexpr (AXPBY) scale_into<V, true>(acc[u], y, sc);
                    store_vec_dword_aligned<V>(y, acc[u]);
                }
            }
        }
    }
}

// ===========================================================================
// Row-split, sequential reduction with coalesced sparse-row caching
// (Section 2.1.3)
// ===========================================================================
//
// 2^logG lanes own a row and V*2^logG dense columns (lane gl owns columns
// [cb*G*V + gl*V, +V)); a wave owns the 64/G consecutive rows of its lane
// groups.  Those rows' (colidx, val) pairs are one contiguous stretch of the
// CSR arrays, so the whole wave stages it in LDS with coalesced loads, kRsSrTile
// pairs at a time (with few lanes per row a group-by-group load would fetch a
// handful of bytes per group).  Every group then walks the cached part of its
// own row and accumulates its own columns: the dense accesses of a group are
// one contiguous 4*V*G-byte piece of a row of X.
// blockIdx.y selects the column block when N > 64*V.

constexpr int kRsSrTile = 512;   // cached pairs per wave and round
// DEPTH (template parameter of the sequential kernels) = dense-row loads a lane keeps in flight.
// More is not always better.  With ascending columns the lanes of a wave, and the waves that
// start together, sweep X from low to high rows in step; every load in flight widens the window
// of X they touch at one time, and once that window outgrows the L2 the hit rate drops (measured
// on 2^20 rows of 27 uniform columns, N = 4: 58 % L2 hits and 224 us at depth 1, 26 % and 373 us
// at depth 4).  Rows that hit in cache anyway want the latency hidden instead (27-point stencil,
// N = 8: 204 us at depth 4, 260 us at depth 1), and so do rows of uneven length.  The host picks.

template <int V, bool XBUF, int DEPTH, bool AXPBY = false, bool RAGGED = false>
__global__ __launch_bounds__(kBlock) void rs_sr_kernel(int M, long long K, int N, int ldx, int ldy, const int* __restrict__ rowptr,
                                                        const int* __restrict__ colidx,
                                                        const float* __restrict__ vals,
                                                        const float* __restrict__ X, float* __restrict__ Y,
                                                        int logG, int cols_per_block, Scaling sc = Scaling{1.0f, 0.0f}) {
    constexpr int T = kRsSrTile;
    __shared__ __align__(16) int s_col[kWavesPerBlock][T];
    __shared__ __align__(16) float s_val[kWavesPerBlock][T];
    const int lane = lane_id();
    const int wib = wave_in_block();
    int* cc = s_col[wib];
    float* cv = s_val[wib];
    const int G = 1 << logG;
    const int gl = lane & (G - 1);
    const int g = lane >> logG;
    const int rows_per_wave = kWave >> logG;

    const LaneColumns mine = lane_columns<V, RAGGED>(blockIdx.y, cols_per_block, gl, N);
    const long long n = mine.first;                              // my first dense column
    const bool col_ok = mine.any;

    const unsigned nwaves = gridDim.x * kWavesPerBlock;
    const unsigned gw = xcd_contiguous(blockIdx.x, gridDim.x) * kWavesPerBlock + wib;
    const unsigned ngroups = ((unsigned)M + rows_per_wave - 1) / rows_per_wave;

    // XBUF: the dense operand is read through a descriptor (its byte offsets fit 32 bits)
    const unsigned long long x_bytes = dense_bytes(K, ldx, N);
    const __amdgpu_buffer_rsrc_t rx = make_buffer(X, XBUF ? x_bytes : 0ull);
    const unsigned n_bytes = (unsigned)n * 4u;

    for (unsigned rg = gw; rg < ngroups; rg += nwaves) {
        const long long row0 = (long long)rg * rows_per_wave;
        const long long row = row0 + g;
        const bool live = row < M;
        unsigned rs = 0, re = 0;
        if (live) { rs = (unsigned)rowptr[row]; re = (unsigned)rowptr[row + 1]; }
        const long long row_end = row0 + rows_per_wave < M ? row0 + rows_per_wave : M;
        const unsigned ps = (unsigned)uniform((int)rs);                  // lane 0 holds row0
        const unsigned pe = (unsigned)uniform(rowptr[row_end]);          // the wave's rows span [ps, pe)
        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.0f;

        for (unsigned ws = ps; ws < pe; ws += (unsigned)T) {
            wave_lds_sync();                    // last round's readers are done
            const unsigned long long bytes = (unsigned long long)(pe - ws) * 4ull;
            const __amdgpu_buffer_rsrc_t rc = make_buffer(colidx + ws, bytes);
            const __amdgpu_buffer_rsrc_t ra = make_buffer(vals + ws, bytes);
#pragma unroll
            for (int k = 0; k < T / kWave; ++k) {
                if (ws + (unsigned)(k * kWave) < pe) {       // wave-uniform
                    const unsigned off = (unsigned)(k * kWave + lane) * 4u;
                    cc[k * kWave + lane] = buffer_stream_i32(rc, off);
                    cv[k * kWave + lane] = buffer_stream_f32(ra, off);
                }
            }
            wave_lds_sync();
            const unsigned we = pe - ws > (unsigned)T ? ws + T : pe;
            const unsigned lo = rs > ws ? rs : ws;
            const unsigned hi = re < we ? re : we;
            if (col_ok) {
                for (unsigned p0 = lo; p0 < hi; p0 += DEPTH) {
                    float x[DEPTH][V]; float a[DEPTH];
#pragma unroll
                    for (int u = 0; u < DEPTH; ++u) {
                        const bool ok = p0 + u < hi;
                        const int e = ok ? (int)(p0 + u - ws) : 0;
                        a[u] = ok ? cv[e] : 0.0f;
                        const unsigned c = (unsigned)cc[e];
                        if constexpr (XBUF) {
                            buffer_load_vec<V>(rx, ok ? c * (unsigned)ldx * 4u + n_bytes : kOutOfRange, x[u]);
                        } else {
                            load_vec_dword_aligned<V>(X + (size_t)(ok ? c : 0u) * ldx + n, x[u]);
#pragma unroll
                            for (int i = 0; i < V; ++i) x[u][i] = ok ? x[u][i] : 0.0f;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < DEPTH; ++u)
#pragma unroll
                        for (int i = 0; i < V; ++i) acc[i] = fmaf(a[u], x[u][i], acc[i]);
                }
            }
        }
        if (live && col_ok) {
            float* y = Y + (size_t)row * ldy + n;
            if constexpr (AXPBY) scale_into<V, true>(acc, y, sc);
            if (AXPBY && RAGGED && mine.skip != 0) {
                // the scaled result depends on the old Y, which the neighbour (another column block, another time)
                // may have replaced: the shared columns are the neighbour's to write
#pragma unroll
                for (int i = 1; i < V; ++i)
                    if (i >= mine.skip) y[i] = acc[i];
            } else {
                store_vec_dword_aligned<V>(y, acc);      // plain product: shared columns hold the same bits in both lanes
            }
        }
    }
}

// Row-split sequential reduction WITHOUT the LDS tile (the kernel Section 2.1.3 compares its
// sparse-row caching against): same row and column mapping as rs_sr_kernel, but every lane of a
// group reads colidx[p] and vals[p] itself, straight from memory, one entry after the other.
// Kept for measurements only.
template <int V>
__global__ __launch_bounds__(kBlock) void rs_sr_direct_kernel(int M, int N, int ldx, int ldy, const int* __restrict__ rowptr,
                                                               const int* __restrict__ colidx,
                                                               const float* __restrict__ vals,
                                                               const float* __restrict__ X, float* __restrict__ Y,
                                                               int logG, int cols_per_block) {
    const int lane = lane_id();
    const int G = 1 << logG;
    const int gl = lane & (G - 1);
    const int g = lane >> logG;
    const int rows_per_wave = kWave >> logG;
    const LaneColumns mine = lane_columns<V, false>(blockIdx.y, cols_per_block, gl, N);
    const long long n = mine.first;
    const bool col_ok = mine.any;
    const unsigned nwaves = gridDim.x * kWavesPerBlock;
    const unsigned gw = xcd_contiguous(blockIdx.x, gridDim.x) * kWavesPerBlock + wave_in_block();
    const unsigned ngroups = ((unsigned)M + rows_per_wave - 1) / rows_per_wave;
    for (unsigned rg = gw; rg < ngroups; rg += nwaves) {
        const long long row = (long long)rg * rows_per_wave + g;
        if (row >= M || !col_ok) continue;
        const int rs = rowptr[row], re = rowptr[row + 1];
        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.0f;
        for (int p = rs; p < re; ++p) {
            const int c = colidx[p];
            const float a = vals[p];
            float x[V];
            load_vec<V>(X + (size_t)c * ldx + n, x);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = fmaf(a, x[i], acc[i]);
        }
        store_vec<V>(Y + (size_t)row * ldy + n, acc);
    }
}

// ===========================================================================
// nnz-balanced kernels: common partition
// ===========================================================================
//
// The paper hands every warp the same count of stored entries (Section 2.1.1).
// Counting only stored entries leaves one hole: a stretch of (nearly) empty
// rows puts an unbounded number of row boundaries into one share.  So the
// unit of work here is the *item* of the merge path of Merrill & Garland, which the
// paper cites as the fine-grained way to balance (Section 1): the list
//     entries of row 0, end of row 0, entries of row 1, end of row 1, ...
// has nnz + M items; row r's entries sit at diagonals
// [r + rowptr[r], r + rowptr[r+1]) and its end marker at r + rowptr[r+1].
// Cutting that list into equal pieces bounds both the entries and the rows
// of a piece.  For matrices without empty stretches it is the paper's fixed
// share of non-zeros up to the few percent that row markers add.
//
// The list is cut into kSubRanges * (number of waves) contiguous chunks; wave w
// takes chunks w, w + nwaves, ... (waves of one XCD hold neighbouring chunks).
// Chunks begin at multiples of a quantum of items and differ by at most one
// quantum: chunk c covers quanta [c*Q/parts, (c+1)*Q/parts) of the Q quanta, so
// no wave stays without work while another holds two quanta.  The split is
// static: one contended atomic costs more than a tile on this machine.  A wave
// finds the first row of a chunk with a 64-way search and then walks.
//
// Rows whose items straddle a chunk boundary (in the sequential kernel: the
// boundary of a lane group's run) are combined with fp32 atomic adds; the
// paper does not say how partial rows of different warps meet.  That needs
// zeros underneath.  A small "prepare" kernel zeroes exactly those rows and no
// others; every other row, empty ones included, is written once with a plain
// store by the chunk that holds its end marker.

constexpr unsigned kSubRanges = 1;

// The even split of the Q quanta into `parts` chunks: chunk c starts at quantum floor(c * Q / parts),
// so chunks differ by at most one quantum and the longer ones are spread over the whole list (put
// first, they would all fall to the first XCDs).  The quotients are formed in fp64: numerators stay
// below 2^53 and a non-integer quotient n / m lies at least 1 / m away from an integer, far more than
// the rounding of one correctly rounded division, so the floors are exact - and much cheaper here
// than 64-bit integer division, which the per-row test of the prepare kernel would pay twice.
struct EvenSplit {
    unsigned Q, parts, shift;     // quanta, chunks, log2 of the quantum
    __device__ __forceinline__ EvenSplit(unsigned items, unsigned parts_, unsigned quantum_log2) {
        const unsigned quantum = 1u << quantum_log2;
        Q = (items >> quantum_log2) + ((items & (quantum - 1)) != 0);
        parts = parts_;
        shift = quantum_log2;
    }
    // first item of chunk c (c may be `parts`: the end of the list, rounded up to a quantum)
    __device__ __forceinline__ unsigned start(unsigned c) const {
        const double n = (double)((unsigned long long)c * Q);
        return (unsigned)(n / (double)parts) << shift;
    }
    // chunk that holds item d: the largest c with floor(c * Q / parts) <= d's quantum
    __device__ __forceinline__ unsigned chunk_of(unsigned d) const {
        const unsigned long long q = d >> shift;
        const double n = (double)((q + 1) * parts - 1);
        return (unsigned)(n / (double)Q);
    }
};

// Zeroes the rows whose items do not all lie in one piece of the partition (beta != 0, the scaled
// variants: multiplies them by beta instead, so that the partial sums added later land on beta * Y).
// The pieces are the `parts` chunks of the even split with quanta of
// 2^quantum_log2 items, cut further into tiles of 2^tile_log2 items counted
// from the chunk's start when tile_log2 >= 0.
// One thread per row for the test (split rows are few: at most two per piece);
// a wave then clears its split rows together, 64 columns per store.
__global__ __launch_bounds__(kBlock) void nb_prepare_kernel(int M, int N, int ldy, const int* __restrict__ rowptr,
                                                             float* __restrict__ Y, unsigned parts, unsigned quantum_log2,
                                                             int tile_log2, float beta) {
    const long long row = (long long)blockIdx.x * kBlock + threadIdx.x;
    bool split = false;
    if (row < M) {
        const unsigned first = (unsigned)row + (unsigned)rowptr[row];       // diagonal of the row's first item
        const unsigned last = (unsigned)row + (unsigned)rowptr[row + 1];    // diagonal of its end marker
        // An empty row is a single item.  Every chunk and tile starts at a multiple of the quantum, so a row
        // whose items lie inside one quantum cannot be split: most rows stop here, before the divisions.
        if (first != last && (first >> quantum_log2) != (last >> quantum_log2)) {
            const EvenSplit es((unsigned)rowptr[M] + (unsigned)M, parts, quantum_log2);
            const unsigned c1 = es.chunk_of(first), c2 = es.chunk_of(last);
            split = c1 != c2;
            if (!split && tile_log2 >= 0) {
                const unsigned start = es.start(c1);
                split = (first - start) >> tile_log2 != (last - start) >> tile_log2;
            }
        }
    }
    if (N <= 8) {                                      // narrow rows: the thread clears its own
        if (split) {
            float* y = Y + (size_t)row * ldy;
            for (int n = 0; n < N; ++n) y[n] = beta != 0.0f ? beta * y[n] : 0.0f;
        }
        return;
    }
    // the wave zeroes its split rows together: lane l clears columns l, l + 64, ...
    const int lane = lane_id();
    const long long row0 = row - lane;
    unsigned long long todo = __ballot(split);
    while (todo) {                                                           // wave-uniform
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        float* y = Y + (size_t)(row0 + src) * ldy;
        for (int n = lane; n < N; n += kWave) y[n] = beta != 0.0f ? beta * y[n] : 0.0f;
    }
}

// The chunks of the calling wave: chunk(s) = s * nwaves + wave id, s < kSubRanges.
struct ChunkPlan {
    unsigned nnz, items, nwaves, gw;
    EvenSplit split;
    __device__ __forceinline__ ChunkPlan(unsigned nnz_, unsigned items_, unsigned nwaves_, unsigned gw_,
                                         unsigned quantum_log2)
        : nnz(nnz_), items(items_), nwaves(nwaves_), gw(gw_), split(items_, nwaves_ * kSubRanges, quantum_log2) {}
    __device__ __forceinline__ bool range(unsigned s, unsigned& d0, unsigned& d1) const {
        const unsigned c = s * nwaves + gw;
        d0 = split.start(c);
        const unsigned e = split.start(c + 1);
        d1 = e < items ? e : items;
        return d0 < d1;
    }
};

__device__ __forceinline__ ChunkPlan plan_chunks(const int* __restrict__ rowptr, int M, unsigned quantum_log2) {
    const unsigned nnz = (unsigned)rowptr[M];
    return ChunkPlan(nnz, nnz + (unsigned)M, gridDim.x * kWavesPerBlock,
                     xcd_contiguous(blockIdx.x, gridDim.x) * kWavesPerBlock + wave_in_block(), quantum_log2);
}
// the same for a workgroup that is number `wg` of `nwg` sharing the list (a mapping of its own, see nb_sr_kernel)
__device__ __forceinline__ ChunkPlan plan_chunks(const int* __restrict__ rowptr, int M, unsigned quantum_log2, unsigned wg,
                                                 unsigned nwg) {
    const unsigned nnz = (unsigned)rowptr[M];
    return ChunkPlan(nnz, nnz + (unsigned)M, nwg * kWavesPerBlock, wg * kWavesPerBlock + wave_in_block(), quantum_log2);
}

// Number of rows whose end marker lies before diagonal d, i.e. rows r with
// r + rowptr[r+1] < d (that key is strictly increasing in r).  64-way search,
// wave-uniform result.
__device__ __forceinline__ int wave_merge_rows_before(const int* __restrict__ rowptr, int M, unsigned d, int lane) {
    int lo = 0, hi = M;   // rows < lo end before d; rows >= hi do not
    while (hi > lo) {
        const int span = hi - lo;
        const int step = (span + 63) >> 6;
        const long long r = (long long)lo + (long long)lane * step;
        bool before = false;
        if (r < hi) before = (unsigned)r + (unsigned)rowptr[r + 1] < d;
        const int cnt = __popcll(__ballot(before));   // probes are monotone: 1...10...0
        if (cnt == 0) {
            hi = lo;
        } else {
            const int nlo = lo + (cnt - 1) * step + 1;
            const int nhi = lo + cnt * step;
            lo = nlo;
            hi = nhi < hi ? nhi : hi;
        }
    }
    return uniform(lo);
}

constexpr unsigned kNoRow = 0xffffffffu;

// ===========================================================================
// nnz-balanced, parallel reduction: vectorized segment reduction (Section 2.1.1)
// ===========================================================================
//
// Tile = W = 64*E items (E = 4*KQ entries per lane).
//   1. Entry 64*e + l of the tile is loaded by lane l (coalesced dword loads),
//      which gathers V dense values for it with one vector load and
//      multiplies.  Consecutive lanes hold consecutive entries, so the gather
//      of a wave touches as few cache lines as the matrix allows.
//   2. The products go through LDS once to change hands: afterwards lane l
//      holds the products of the E consecutive entries E*l ... and reduces them
//      in order in registers.
//   3. Row ends are scattered into LDS as marks (row i ends after entry q), so
//      a lane sees its own boundaries with one 16-byte LDS read.  A lane
//      without a boundary contributes its whole sum to the row that is open
//      across lanes; a lane with boundaries closes that open row with its
//      leading part, finishes the rows that lie inside it, and opens a new
//      segment with its trailing part.
//   4. The open row's running sum across lanes is the paper's segment
//      reduction: the wave64 DPP scan that adds a partner lane's value only
//      when no row boundary lies in between (one scan per tile instead of
//      one per 64 entries).
//   5. The rows that end in a tile are consecutive, so finished sums are put
//      into LDS by row and written out together: lane l stores row is + l.
//      Rows without entries keep the zero the buffer was cleared to.  The
//      store of the first 64 rows is issued a tile later, behind that tile's
//      loads.
//   6. The sum still open at the end of a tile is handed to the chunk's next
//      tile in a register; only the two ends of a chunk can need an atomic add.
//
// Memory operations inside the tile loop are unconditional: loads and the row
// store go through buffer descriptors, and a lane that has nothing to load or
// write pushes its offset out of range (the buffer unit returns zero / drops
// the store and touches no memory).  With no branch around them the
// outstanding-operation counter can be waited on exactly, which is what lets
// the next tile's loads stay in flight while this tile is reduced.
// blockIdx.y selects the group of V dense columns (N > V: one pass each).

template <int V, int KQ, bool AXPBY = false>
__global__ __launch_bounds__(kBlock) void nb_pr_tiled_kernel(int M, long long K, int N, int ldx, int ldy, const int* __restrict__ rowptr,
                                                        const int* __restrict__ colidx,
                                                        const float* __restrict__ vals,
                                                        const float* __restrict__ X, float* __restrict__ Y,
                                                        Scaling sc = Scaling{1.0f, 0.0f}) {
    constexpr int E = 4 * KQ;
    constexpr int W = kWave * E;
    // accessed 16 bytes at a time: every wave's part starts on a 16-byte boundary ((W + 4) * 4 and W * V * 4 are multiples of 16)
    __shared__ __align__(16) unsigned s_bnd[kWavesPerBlock][W + 4];   // [W]: rows that end before the tile's first entry
    __shared__ __align__(16) float s_buf[kWavesPerBlock][W * V];      // products, then the tile's row results
    const int lane = lane_id();
    const int wib = wave_in_block();
    unsigned* bnd = s_bnd[wib];
    float* buf = s_buf[wib];
    const int n0 = blockIdx.y * V;

    const ChunkPlan plan = plan_chunks(rowptr, M, 6);        // quanta of one wave's width
    const unsigned nnz = plan.nnz;
    const unsigned long long y_elems = dense_bytes(M, ldy, N) / 4ull;
    // V = 8: the lane's second four columns start here.  N = 5, 6, 7 (one pass, n0 = 0): at N - 4, overlapping
    // the first four; the shared columns get the same sums twice and are added to memory once.
    const int second = (V == 8 && N - n0 < 8) ? N - n0 - 4 : 4;

    auto add_to_row = [&](float* y, const float (&v)[V]) {
        if constexpr (V == 8) atomic_add_halves(y, v, second); else atomic_add_vec<V>(y, v);
    };

    for (unsigned sub = 0; sub < kSubRanges; ++sub) {
    unsigned d0, d1;
    if (!plan.range(sub, d0, d1)) continue;

    if (nnz == 0) {
        // nothing stored: every item is a row end; my rows are [d0, d1)
        float zero[V];
#pragma unroll
        for (int i = 0; i < V; ++i) zero[i] = 0.0f;
        for (unsigned r = d0 + lane; r < d1; r += kWave) {
            float* y = Y + (size_t)r * ldy + n0;
            float out[V];
#pragma unroll
            for (int i = 0; i < V; ++i) out[i] = 0.0f;
            if constexpr (AXPBY) scale_into<V, true>(out, y, sc, second);
            store_vec_dword_aligned<V>(y, out, second);
        }
        continue;
    }

    int is = wave_merge_rows_before(rowptr, M, d0, lane);   // rows that ended before my chunk
    unsigned js = d0 - (unsigned)is;                        // entries consumed before my chunk
    // the first row to end in my chunk started before it?  then its sum is shared with another wave
    const int r_first = is;
    const bool first_split = is < M && (unsigned)is + (unsigned)rowptr[is] < d0;

    // entries of a tile starting at entry `from`: at most W.  The descriptor ends at the arrays' end,
    // so lanes past it load nothing; `on` = false switches the whole load off.
    auto load_entries = [&](unsigned from, bool on, int (&c)[E], float (&a)[E]) {
        const unsigned long long bytes = on ? (unsigned long long)(nnz - from) * 4ull : 0ull;
        const __amdgpu_buffer_rsrc_t rc = make_buffer(colidx + from, bytes);
        const __amdgpu_buffer_rsrc_t ra = make_buffer(vals + from, bytes);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const unsigned off = (unsigned)(e * kWave + lane) * 4u;
            c[e] = (int)__builtin_amdgcn_raw_buffer_load_b32(rc, off, 0, 2);
            a[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ra, off, 0, 2));
        }
    };
    // start and end offset of row `first + lane`; rows past the last one read as 0, 0
    auto load_row_bounds = [&](int first, bool on, unsigned& start, unsigned& end) {
        const unsigned long long bytes = (on && first < M) ? (unsigned long long)(M + 1 - first) * 4ull : 0ull;
        const __amdgpu_buffer_rsrc_t rr = make_buffer(rowptr + first, bytes);
        typedef unsigned u2 __attribute__((ext_vector_type(2)));
        const u2 t = __builtin_amdgcn_raw_buffer_load_b64(rr, (unsigned)lane * 4u, 0, 0);
        start = t.x; end = t.y;
    };
    // the dense operand: byte offsets of X rows fit 32 bits unless X is 4 GB or more
    const unsigned long long x_bytes = dense_bytes(K, ldx, N);
    const bool x_small = x_bytes <= 0xffffffffull;
    const __amdgpu_buffer_rsrc_t rx = make_buffer(X + n0, x_small ? x_bytes - (unsigned)n0 * 4ull : 0ull);

    float carry[V];      // running sum of the row that is open at the tile boundary (wave-uniform)
#pragma unroll
    for (int i = 0; i < V; ++i) carry[i] = 0.0f;

    // two register sets take turns: while one tile is reduced the other set receives the next tile
    int cA[E], cB[E]; float aA[E], aB[E]; unsigned wA, wB, w_unused;
    load_row_bounds(is, true, w_unused, wA);
    load_entries(js, true, cA, aA);
    unsigned ds = d0;

    // The first 64 row results of a tile are stored one tile later, after the next tile's loads have been issued:
    // the memory pipeline retires loads and stores in issue order, so a store in front of the gathers would put
    // its own round trip into their wait.
    float pending_val[V];
    unsigned pending_off = kOutOfRange;
    unsigned long long pending_first = 0ull;             // first element of the rows the pending store addresses
#pragma unroll
    for (int i = 0; i < V; ++i) pending_val[i] = 0.0f;
    auto rows_descriptor = [&](unsigned long long first_elem) {
        const unsigned long long left = first_elem < y_elems ? (y_elems - first_elem) * 4ull : 0ull;
        return __builtin_amdgcn_make_buffer_rsrc((void*)(Y + first_elem), 0, left > 0xffffffffull ? 0xffffffffu : (unsigned)left,
                                                 kBufferFlags);
    };
    auto store_pending = [&]() {
        buffer_store_vec<V>(rows_descriptor(pending_first), pending_off, pending_val, second);
        pending_off = kOutOfRange;
    };

    // one tile: consumes (c, a, w_end), leaves the next tile's loads in flight in (c2, a2, w_end2)
    auto do_tile = [&](int (&c)[E], float (&a)[E], unsigned w_end, int (&c2)[E], float (&a2)[E], unsigned& w_end2) {
        const unsigned de = (d1 - ds > (unsigned)W) ? ds + W : d1;

        // ---- row ends of this tile -> LDS marks
        wave_lds_sync();                                   // the previous tile's readers are done
#pragma unroll
        for (int k = 0; k < KQ; ++k)
            *reinterpret_cast<uint4*>(bnd + E * lane + 4 * k) = make_uint4(kNoRow, kNoRow, kNoRow, kNoRow);
        if (lane == 0) bnd[W] = kNoRow;
        wave_lds_sync();
        int ie = is;
        // marks the rows of one batch of 64 candidates that end in the tile; returns how many did
        auto mark_row_ends = [&](int m, unsigned end) {
            const long long r = (long long)is + m * kWave + lane;
            const bool ends = r < M && (unsigned)r + end < de;     // the row's end marker is inside the tile
            if (ends) {
                const unsigned q = end - js;               // it ends after entry q-1 of the tile
                atomicMin(bnd + (q ? q - 1 : (unsigned)W), (unsigned)(r - is));
            }
            return (int)__popcll(__ballot(ends));
        };
        int cnt = mark_row_ends(0, w_end);                 // the first 64 candidates were loaded a tile ago
        ie += cnt;
        if (cnt == kWave) {
            // a tile crowded with row ends (at most W of them): fetch all remaining candidates at once
            unsigned ms[E - 1], me[E - 1];
#pragma unroll
            for (int m = 1; m < E; ++m) load_row_bounds(is + m * kWave, true, ms[m - 1], me[m - 1]);
#pragma unroll
            for (int m = 1; m < E; ++m) {
                if (cnt == kWave) { cnt = mark_row_ends(m, me[m - 1]); ie += cnt; }
            }
        }
        const unsigned je = de - (unsigned)ie;             // entries [js, je) belong to the tile
        const int nE = (int)(je - js);
        const int nrows = ie - is;                         // rows [is, ie) end in the tile
        wave_lds_sync();

        // ---- gather for this tile, then the next tile's loads (they stay in flight during the reduction)
        float x[E][V];
        if (x_small) {
#pragma unroll
            for (int e = 0; e < E; ++e)
                buffer_load_vec<V>(rx, e * kWave + lane < nE ? (unsigned)c[e] * (unsigned)ldx * 4u : kOutOfRange, x[e], second);
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) load_vec_dword_aligned<V>(X + (size_t)(e * kWave + lane < nE ? c[e] : 0) * ldx + n0, x[e], second);
        }
        {
            const bool more = d1 - ds > (unsigned)W;       // past the chunk's last tile the loads are switched off
            load_row_bounds(ie, more, w_unused, w_end2);
            load_entries(je, more, c2, a2);
        }
        store_pending();                                   // the previous tile's rows

        // ---- products change hands through LDS: entry 64e+l -> lane (64e+l)/E
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float p[V];
            const bool mine = e * kWave + lane < nE;
#pragma unroll
            for (int i = 0; i < V; ++i) p[i] = mine ? a[e] * x[e][i] : 0.0f;
            store_vec<V>(buf + (size_t)(e * kWave + lane) * V, p);
        }
        wave_lds_sync();
        const unsigned b_in = bnd[W];
        unsigned b[E];
#pragma unroll
        for (int k = 0; k < KQ; ++k) {
            const uint4 t = *reinterpret_cast<const uint4*>(bnd + E * lane + 4 * k);
            b[4 * k] = t.x; b[4 * k + 1] = t.y; b[4 * k + 2] = t.z; b[4 * k + 3] = t.w;
        }
        float pr[E][V];
#pragma unroll
        for (int e = 0; e < E; ++e) load_vec<V>(buf + (size_t)(E * lane + e) * V, pr[e]);
        wave_lds_sync();                                   // products are in registers: the buffer is free

        // ---- the tile's row results: cleared, so rows without entries come out as zeros
        for (int k = 0; k * kWave < nrows; ++k) {
            float zero[V];
#pragma unroll
            for (int i = 0; i < V; ++i) zero[i] = 0.0f;
            store_vec<V>(buf + (size_t)(k * kWave + lane) * V, zero);
        }
        wave_lds_sync();
        // rows that end before the tile's first entry take the sum carried in
        if (b_in != kNoRow) {
            if (lane == 0) store_vec<V>(buf + (size_t)b_in * V, carry);
#pragma unroll
            for (int i = 0; i < V; ++i) carry[i] = 0.0f;
        }

        // ---- in-lane reduction over my E consecutive entries
        float s[V], head[V];
        unsigned head_row = kNoRow;                        // kNoRow: no boundary inside this lane
#pragma unroll
        for (int i = 0; i < V; ++i) { s[i] = lane == 0 ? carry[i] : 0.0f; head[i] = 0.0f; }
#pragma unroll
        for (int e = 0; e < E; ++e) {
#pragma unroll
            for (int i = 0; i < V; ++i) s[i] += pr[e][i];
            if (b[e] != kNoRow) {
                if (head_row == kNoRow) {
                    head_row = b[e];
#pragma unroll
                    for (int i = 0; i < V; ++i) head[i] = s[i];
                } else {
                    store_vec<V>(buf + (size_t)b[e] * V, s);   // a row that begins and ends inside this lane
                }
#pragma unroll
                for (int i = 0; i < V; ++i) s[i] = 0.0f;
            }
        }

        // ---- the open row across lanes: segments start at lanes that hold a boundary
        const bool flagged = head_row != kNoRow;
        const int head_lane = (int)wave_max_scan(flagged ? (unsigned)lane : 0u);
        segmented_scan<V>(s, lane - head_lane, lane);      // s: sum of the open row up to and including my lane
        {
            float closing[V];
#pragma unroll
            for (int i = 0; i < V; ++i) closing[i] = dpp_or_zero<kDppWaveShr1, 0xf>(s[i]) + head[i];
            if (flagged) store_vec<V>(buf + (size_t)head_row * V, closing);
        }
#pragma unroll
        for (int i = 0; i < V; ++i) carry[i] = read_lane(s[i], kWave - 1);
        wave_lds_sync();

        // ---- write the rows [is, ie) out, lane l row is + l: the first 64 with one unconditional
        //      buffer store, further batches (tiles crowded with short rows) in a loop
        {
            const unsigned long long first_elem = (unsigned long long)is * (unsigned)ldy + (unsigned)n0;
            __amdgpu_buffer_rsrc_t yrows = rows_descriptor(first_elem);
            auto write_rows = [&](int k) {
                const int t = k * kWave + lane;                     // local row
                float val[V];
                load_vec<V>(buf + (size_t)t * V, val);
                const bool live = t < nrows;
                const bool shared = first_split && is + t == r_first;   // finished by an atomic add instead
                const unsigned off = (live && !shared) ? (unsigned)t * (unsigned)ldy * 4u : kOutOfRange;
                if constexpr (AXPBY) {
                    if (live && shared) {
#pragma unroll
                        for (int i = 0; i < V; ++i) val[i] *= sc.alpha;          // lands on beta * Y (prepare)
                    } else {
                        scale_into<V>(val, yrows, off, sc, second);
                    }
                }
                if (k == 0) {
                    pending_first = first_elem; pending_off = off;
#pragma unroll
                    for (int i = 0; i < V; ++i) pending_val[i] = val[i];
                } else {
                    buffer_store_vec<V>(yrows, off, val, second);
                }
                if (live && shared) add_to_row(Y + (size_t)(is + t) * ldy + n0, val);
            };
            write_rows(0);
            for (int k = 1; k * kWave < nrows; ++k) write_rows(k);
        }

        is = ie;
        js = je;
        ds += W;
    };
    while (ds < d1) {
        do_tile(cA, aA, wA, cB, aB, wB);
        if (ds >= d1) break;
        do_tile(cB, aB, wB, cA, aA, wA);
    }

    store_pending();                                       // the last tile's rows
    // the row still open at the end of my chunk is finished by another wave
    bool any = false;
#pragma unroll
    for (int i = 0; i < V; ++i) any |= carry[i] != 0.0f;
    if constexpr (AXPBY) {
#pragma unroll
        for (int i = 0; i < V; ++i) carry[i] *= sc.alpha;
    }
    if (any && lane == 0 && is < M) add_to_row(Y + (size_t)is * ldy + n0, carry);
    }   // next chunk
}

// ===========================================================================
// nnz-balanced, parallel reduction with the entry stream decoupled from the rows
// ===========================================================================
//
// The kernel above cuts a chunk into tiles of W merge-path items, so where the entries of tile t + 1 begin is
// known only when the row ends of tile t have been counted: its gathers cannot be requested before the row
// logic of tile t is through, and a wave spends that logic with no gather in flight.  Here the chunk (still an
// equal share of merge-path items, found by two 64-way searches in lock-step) is walked in BLOCKS of W consecutive
// ENTRIES counted from the chunk's first entry, so every block's address is known from the start:
//   * everything a block needs from memory is requested one block ahead: while the rows of block k are finished,
//     the gathers of block k + 1 and the entries of block k + 2 are in flight (the entries land in registers of
//     their own and are moved when they have arrived, so the loop needs no unrolling);
//   * the products of a block change hands through LDS as before (lane l ends up with E consecutive products)
//     and stay in registers while the rows that end inside the block are finished in STEPS: a step takes up to W
//     row ends (the LDS marks and the staged row results are sized for that) and the entries up to the end of the
//     last of them, or up to the block's end when fewer than W rows end in the block - the usual case, one step
//     per block.  A stretch of empty rows simply takes more steps; entries outside the step's range are masked;
//   * per step everything else is the scheme of the kernel above: row-end marks in LDS, in-lane sums of E
//     consecutive products, one segmented DPP scan over the lanes' open-row partials (Section 2.1.1), results
//     staged by row and stored 64 rows at a time, the open row's sum carried in a register.
// The row-bound window of the next step is requested before the next entries, so waiting for it does not wait
// for them (loads return in issue order).

// Rows that ended before diagonal da, and before db (both searches of wave_merge_rows_before in lock-step: their
// probes are in flight together, so the second costs no further round trips).
__device__ __forceinline__ void wave_merge_rows_before2(const int* __restrict__ rowptr, int M, unsigned da, unsigned db,
                                                        int lane, int& ra, int& rb) {
    int lo[2] = {0, 0}, hi[2] = {M, M};
    const unsigned d[2] = {da, db};
    while (hi[0] > lo[0] || hi[1] > lo[1]) {
        int step[2], v[2];
        long long r[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            step[k] = (hi[k] - lo[k] + 63) >> 6;
            r[k] = (long long)lo[k] + (long long)lane * step[k];
            v[k] = (hi[k] > lo[k] && r[k] < hi[k]) ? rowptr[r[k] + 1] : 0;
        }
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            if (hi[k] > lo[k]) {                                   // wave-uniform
                const bool before = r[k] < hi[k] && (unsigned)r[k] + (unsigned)v[k] < d[k];
                const int cnt = __popcll(__ballot(before));       // probes are monotone: 1...10...0
                if (cnt == 0) {
                    hi[k] = lo[k];
                } else {
                    const int nlo = lo[k] + (cnt - 1) * step[k] + 1;
                    const int nhi = lo[k] + cnt * step[k];
                    lo[k] = nlo;
                    hi[k] = nhi < hi[k] ? nhi : hi[k];
                }
            }
        }
    }
    ra = uniform(lo[0]);
    rb = uniform(lo[1]);
}

// SERIAL_SCAN (a comparison kernel for Section 2.1.1, not used by the library's own choices): the lanes' open-row
// partial sums meet through a serial segmented prefix sum - they are put into LDS and one lane adds them up in
// lane order, starting afresh at every lane that holds a row boundary - instead of the DPP network.  Everything
// else, the balanced split included, is the same, so the difference in time is the vectorized reduction's.
template <int V, int KQ, bool AXPBY = false, bool SERIAL_SCAN = false>
__global__ __launch_bounds__(kBlock) void nb_pr_kernel(int M, long long K, int N, int ldx, int ldy, const int* __restrict__ rowptr,
                                                        const int* __restrict__ colidx,
                                                        const float* __restrict__ vals,
                                                        const float* __restrict__ X, float* __restrict__ Y,
                                                        Scaling sc = Scaling{1.0f, 0.0f}) {
    constexpr int E = 4 * KQ;
    constexpr int W = kWave * E;
    __shared__ __align__(16) unsigned s_bnd[kWavesPerBlock][W + 4];   // [W]: rows that end before the step's first entry
    __shared__ __align__(16) float s_buf[kWavesPerBlock][W * V];      // products, then a step's row results
    __shared__ __align__(16) float s_scan[SERIAL_SCAN ? kWavesPerBlock : 1][SERIAL_SCAN ? kWave * (V + 1) : 1];   // serial scan only
    const int lane = lane_id();
    const int wib = wave_in_block();
    unsigned* bnd = s_bnd[wib];
    float* buf = s_buf[wib];
    const int n0 = blockIdx.y * V;

    const ChunkPlan plan = plan_chunks(rowptr, M, 6);        // quanta of one wave's width
    const unsigned nnz = plan.nnz;
    const unsigned long long y_elems = dense_bytes(M, ldy, N) / 4ull;
    // V = 8: the lane's second four columns start here (N = 5, 6, 7: at N - 4, overlapping the first four)
    const int second = (V == 8 && N - n0 < 8) ? N - n0 - 4 : 4;

    auto add_to_row = [&](float* y, const float (&v)[V]) {
        if constexpr (V == 8) atomic_add_halves(y, v, second); else atomic_add_vec<V>(y, v);
    };

    for (unsigned sub = 0; sub < kSubRanges; ++sub) {
    unsigned d0, d1;
    if (!plan.range(sub, d0, d1)) continue;

    if (nnz == 0) {
        // nothing stored: every item is a row end; my rows are [d0, d1)
        for (unsigned r = d0 + lane; r < d1; r += kWave) {
            float* y = Y + (size_t)r * ldy + n0;
            float out[V];
#pragma unroll
            for (int i = 0; i < V; ++i) out[i] = 0.0f;
            if constexpr (AXPBY) scale_into<V, true>(out, y, sc, second);
            store_vec_dword_aligned<V>(y, out, second);
        }
        continue;
    }

    // my chunk: rows [is, ie1) end in it, entries [js0, je1) lie in it
    int is, ie1;
    wave_merge_rows_before2(rowptr, M, d0, d1, lane, is, ie1);
    const unsigned js0 = d0 - (unsigned)is;
    const unsigned je1 = d1 - (unsigned)ie1;
    unsigned js = js0;
    // the first row to end in my chunk started before it?  then its sum is shared with another wave
    const int r_first = is;
    const bool first_split = is < M && (unsigned)is + (unsigned)rowptr[is] < d0;

    // entries of block k of my chunk (lane l: entries 64 e + l of the block); nothing past the chunk's last entry
    // One descriptor pair for the whole chunk (a wave's share of a matrix the library takes stays far below the
    // 4 GB a descriptor spans); a block is a byte offset into it, kept in a VGPR and advanced by 4 W per block.
    const unsigned long long chunk_bytes = ((unsigned long long)je1 - js0) * 4ull;
    const __amdgpu_buffer_rsrc_t rc = make_buffer(colidx + js0, chunk_bytes);
    const __amdgpu_buffer_rsrc_t ra = make_buffer(vals + js0, chunk_bytes);
    auto load_entries = [&](unsigned k, int (&c)[E], float (&a)[E]) {
        // past the chunk's last block every offset is out of range: nothing is loaded (k * W * 4 cannot wrap: k <= nb + 1)
        const unsigned base = (unsigned long long)k * W * 4ull < chunk_bytes ? k * (unsigned)(W * 4) + (unsigned)lane * 4u : kOutOfRange;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const unsigned off = base == kOutOfRange ? kOutOfRange : base + (unsigned)(e * kWave) * 4u;
            c[e] = (int)__builtin_amdgcn_raw_buffer_load_b32(rc, off, 0, 2);
            a[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ra, off, 0, 2));
        }
    };
    // the dense operand: byte offsets of X rows fit 32 bits unless X is 4 GB or more
    const unsigned long long x_bytes = dense_bytes(K, ldx, N);
    const bool x_small = x_bytes <= 0xffffffffull;
    const __amdgpu_buffer_rsrc_t rx = make_buffer(X + n0, x_small ? x_bytes - (unsigned)n0 * 4ull : 0ull);
    // one vector gather per entry of block k, from the columns that load_entries(k) brought
    // Entries past the chunk's end were loaded as column 0, value 0: their gathers read row 0 of X (in range: the
    // matrix has entries, so K >= 1) and their products are masked, so the gathers need no mask of their own.
    // Row offsets: a shift when the row pitch is a power of two (packed X at N = 1, 2: the 32-bit multiply runs at
    // a quarter of the rate of other vector instructions), checked once.
    const unsigned pitch = (unsigned)ldx * 4u;
    const int pitch_shift = (pitch & (pitch - 1u)) == 0u ? __builtin_ctz(pitch) : -1;
    auto gather = [&](unsigned k, const int (&c)[E], float (&x)[E][V]) {
        if ((unsigned long long)k * W * 4ull >= chunk_bytes && chunk_bytes != 0ull) {
            // no such block: nothing to request (the loop's last iteration)
#pragma unroll
            for (int e = 0; e < E; ++e)
#pragma unroll
                for (int i = 0; i < V; ++i) x[e][i] = 0.0f;
        } else if (x_small) {
            if (pitch_shift >= 0) {
#pragma unroll
                for (int e = 0; e < E; ++e) buffer_load_vec<V>(rx, (unsigned)c[e] << pitch_shift, x[e], second);
            } else {
#pragma unroll
                for (int e = 0; e < E; ++e) buffer_load_vec<V>(rx, (unsigned)c[e] * pitch, x[e], second);
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e)
                load_vec_dword_aligned<V>(X + (size_t)c[e] * ldx + n0, x[e], second);
        }
    };
    // end offset of row `first + lane` (rows past the last one read as 0)
    auto load_row_ends = [&](int first, bool on, unsigned& end) {
        const unsigned long long bytes = (on && first < M) ? (unsigned long long)(M + 1 - first) * 4ull : 0ull;
        const __amdgpu_buffer_rsrc_t rr = make_buffer(rowptr + (bytes ? first : 0), bytes);
        end = __builtin_amdgcn_raw_buffer_load_b32(rr, (unsigned)(lane + 1) * 4u, 0, 0);
    };

    float carry[V];      // running sum of the row that is open at the step boundary (wave-uniform)
#pragma unroll
    for (int i = 0; i < V; ++i) carry[i] = 0.0f;

    // The first 64 row results of a step are stored one step later, behind the loads issued meanwhile (the memory
    // pipeline retires loads and stores in issue order: a store in front of the gathers adds its round trip to their wait).
    float pending_val[V];
    unsigned pending_off = kOutOfRange;
    unsigned long long pending_first = 0ull;             // first element of the rows the pending store addresses
#pragma unroll
    for (int i = 0; i < V; ++i) pending_val[i] = 0.0f;
    auto rows_descriptor = [&](unsigned long long first_elem) {
        const unsigned long long left = first_elem < y_elems ? (y_elems - first_elem) * 4ull : 0ull;
        return __builtin_amdgcn_make_buffer_rsrc((void*)(Y + first_elem), 0, left > 0xffffffffull ? 0xffffffffu : (unsigned)left,
                                                 kBufferFlags);
    };
    auto store_pending = [&]() {
        buffer_store_vec<V>(rows_descriptor(pending_first), pending_off, pending_val, second);
        pending_off = kOutOfRange;
    };

    int c[E]; float a[E], x[E][V];                        // the block whose gathers are in flight
    int lc[E]; float la[E];                               // landing registers of the next block's entries
    unsigned w_end;                                       // end offsets of rows is .. is + 63 (lane l: row is + l)
    load_entries(0, lc, la);
    load_row_ends(is, is < ie1, w_end);
#pragma unroll
    for (int e = 0; e < E; ++e) { c[e] = lc[e]; a[e] = la[e]; }
    load_entries(1, lc, la);
    gather(0, c, x);

    // state of the step in flight between its two halves
    int ie = is, nrows = 0;
    unsigned je = js, blk_start = js0, blk_end = js0;
    bool capped = false;

    // first half of a step: which rows end in it, their marks, the next step's row window
    auto step_rows = [&]() {
        wave_lds_sync();                                   // the previous step's readers are done
#pragma unroll
        for (int k = 0; k < KQ; ++k)
            *reinterpret_cast<uint4*>(bnd + E * lane + 4 * k) = make_uint4(kNoRow, kNoRow, kNoRow, kNoRow);
        if (lane == 0) bnd[W] = kNoRow;
        wave_lds_sync();
        const unsigned js_l = js - blk_start;              // the step's first entry, counted from the block's start
        ie = is;
        // marks the rows of one batch of 64 candidates that end in this block (and in my chunk); returns how many did
        auto mark_row_ends = [&](int m, unsigned end) {
            const long long r = (long long)is + m * kWave + lane;
            const bool ends = r < ie1 && end <= blk_end;
            if (ends) {
                const unsigned q = end - blk_start;        // it ends after entry q-1 of the block; q >= js_l
                atomicMin(bnd + (q > js_l ? q - 1 : (unsigned)W), (unsigned)(r - is));
            }
            return (int)__popcll(__ballot(ends));
        };
        int cnt = mark_row_ends(0, w_end);                 // the first 64 candidates were loaded a step ago
        ie += cnt;
        unsigned last_end = 0;
        if (cnt == kWave) {
            // crowded with row ends: fetch all remaining candidates of the step at once
            unsigned me[E - 1];
#pragma unroll
            for (int m = 1; m < E; ++m) load_row_ends(is + m * kWave, true, me[m - 1]);
#pragma unroll
            for (int m = 1; m < E; ++m) {
                if (cnt == kWave) { cnt = mark_row_ends(m, me[m - 1]); ie += cnt; }
            }
            last_end = (unsigned)read_lane((int)me[E - 2], kWave - 1);      // end of row is + W - 1
        }
        nrows = ie - is;
        capped = nrows == W;                               // more rows may end in this block: another step
        je = capped ? last_end : blk_end;                  // capped: up to the end of the last row taken
        load_row_ends(ie, ie < ie1, w_end);                // candidates of the next step
    };

    // second half: reduce the step's entries, finish its rows
    auto step_sums = [&](const float (&pr)[E][V]) {
        store_pending();                                   // the previous step's rows
        wave_lds_sync();                                   // marks are in place
        const int js_l = (int)(js - blk_start), je_l = (int)(je - blk_start);
        const unsigned b_in = bnd[W];
        unsigned b[E];
#pragma unroll
        for (int k = 0; k < KQ; ++k) {
            const uint4 t = *reinterpret_cast<const uint4*>(bnd + E * lane + 4 * k);
            b[4 * k] = t.x; b[4 * k + 1] = t.y; b[4 * k + 2] = t.z; b[4 * k + 3] = t.w;
        }
        // ---- the step's row results: cleared, so rows without entries come out as zeros
        for (int k = 0; k * kWave < nrows; ++k) {
            float zero[V];
#pragma unroll
            for (int i = 0; i < V; ++i) zero[i] = 0.0f;
            store_vec<V>(buf + (size_t)(k * kWave + lane) * V, zero);
        }
        wave_lds_sync();
        // rows that end before the step's first entry take the sum carried in
        if (b_in != kNoRow) {
            if (lane == 0) store_vec<V>(buf + (size_t)b_in * V, carry);
#pragma unroll
            for (int i = 0; i < V; ++i) carry[i] = 0.0f;
        }

        // ---- in-lane reduction over my E consecutive entries (those of this step)
        float s[V], head[V];
        unsigned head_row = kNoRow;                        // kNoRow: no boundary inside this lane
#pragma unroll
        for (int i = 0; i < V; ++i) { s[i] = lane == 0 ? carry[i] : 0.0f; head[i] = 0.0f; }
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int pos = E * lane + e;
            const bool in = pos >= js_l && pos < je_l;
#pragma unroll
            for (int i = 0; i < V; ++i) s[i] += in ? pr[e][i] : 0.0f;
            if (b[e] != kNoRow) {
                if (head_row == kNoRow) {
                    head_row = b[e];
#pragma unroll
                    for (int i = 0; i < V; ++i) head[i] = s[i];
                } else {
                    store_vec<V>(buf + (size_t)b[e] * V, s);   // a row that begins and ends inside this lane
                }
#pragma unroll
                for (int i = 0; i < V; ++i) s[i] = 0.0f;
            }
        }

        // ---- the open row across lanes: segments start at lanes that hold a boundary
        const bool flagged = head_row != kNoRow;
        if constexpr (SERIAL_SCAN) {
            float* sc_val = s_scan[wib];                   // 64 x V partial sums, then 64 flags
            float* sc_flag = sc_val + kWave * V;
#pragma unroll
            for (int i = 0; i < V; ++i) sc_val[lane * V + i] = s[i];
            sc_flag[lane] = flagged ? 1.0f : 0.0f;
            wave_lds_sync();
            if (lane == 0) {
                float run[V];
#pragma unroll
                for (int i = 0; i < V; ++i) run[i] = 0.0f;
                for (int l = 0; l < kWave; ++l) {          // one lane, lane order: a boundary starts a new sum
                    const bool start = sc_flag[l] != 0.0f;
#pragma unroll
                    for (int i = 0; i < V; ++i) {
                        run[i] = (start ? 0.0f : run[i]) + sc_val[l * V + i];
                        sc_val[l * V + i] = run[i];
                    }
                }
            }
            wave_lds_sync();
#pragma unroll
            for (int i = 0; i < V; ++i) s[i] = sc_val[lane * V + i];
        } else {
            const int head_lane = (int)wave_max_scan(flagged ? (unsigned)lane : 0u);
            segmented_scan<V>(s, lane - head_lane, lane);  // s: sum of the open row up to and including my lane
        }
        {
            float closing[V];
#pragma unroll
            for (int i = 0; i < V; ++i) closing[i] = dpp_or_zero<kDppWaveShr1, 0xf>(s[i]) + head[i];
            if (flagged) store_vec<V>(buf + (size_t)head_row * V, closing);
        }
#pragma unroll
        for (int i = 0; i < V; ++i) carry[i] = read_lane(s[i], kWave - 1);
        wave_lds_sync();

        // ---- write the rows [is, ie) out, lane l row is + l: the first 64 with one unconditional
        //      buffer store (issued a step later), further batches in a loop
        {
            const unsigned long long first_elem = (unsigned long long)is * (unsigned)ldy + (unsigned)n0;
            __amdgpu_buffer_rsrc_t yrows = rows_descriptor(first_elem);
            auto write_rows = [&](int k) {
                const int t = k * kWave + lane;                     // local row
                float val[V];
                load_vec<V>(buf + (size_t)t * V, val);
                const bool live = t < nrows;
                const bool shared = first_split && is + t == r_first;   // finished by an atomic add instead
                const unsigned off = (live && !shared) ? (unsigned)t * (unsigned)ldy * 4u : kOutOfRange;
                if constexpr (AXPBY) {
                    if (live && shared) {
#pragma unroll
                        for (int i = 0; i < V; ++i) val[i] *= sc.alpha;          // lands on beta * Y (prepare)
                    } else {
                        scale_into<V>(val, yrows, off, sc, second);
                    }
                }
                if (k == 0) {
                    pending_first = first_elem; pending_off = off;
#pragma unroll
                    for (int i = 0; i < V; ++i) pending_val[i] = val[i];
                } else {
                    buffer_store_vec<V>(yrows, off, val, second);
                }
                if (live && shared) add_to_row(Y + (size_t)(is + t) * ldy + n0, val);
            };
            write_rows(0);
            for (int k = 1; k * kWave < nrows; ++k) write_rows(k);
        }
        is = ie;
        js = je;
    };

    const unsigned nblocks = (je1 - js0 + (unsigned)W - 1) / (unsigned)W;
    const unsigned nb = nblocks ? nblocks : 1u;            // a chunk without entries still has its row ends to finish
    for (unsigned k = 0; k < nb; ++k) {
        blk_start = js0 + k * (unsigned)W;                 // == js: the previous block was consumed to its end
        blk_end = (je1 - blk_start > (unsigned)W) ? blk_start + (unsigned)W : je1;
        // ---- products of block k change hands through LDS: entry 64e+l of the block -> lane (64e+l)/E
        const int nE = (int)(blk_end - blk_start);
        wave_lds_sync();                                   // the previous step's readers of the buffer are done
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float p[V];
            const bool mine = e * kWave + lane < nE;
#pragma unroll
            for (int i = 0; i < V; ++i) p[i] = mine ? a[e] * x[e][i] : 0.0f;
            store_vec<V>(buf + (size_t)(e * kWave + lane) * V, p);
        }
        wave_lds_sync();
        float pr[E][V];
#pragma unroll
        for (int e = 0; e < E; ++e) load_vec<V>(buf + (size_t)(E * lane + e) * V, pr[e]);
        // ---- block k + 1's entries have landed: request its gathers and block k + 2's entries; both stay in
        //      flight while the rows of block k are finished
#pragma unroll
        for (int e = 0; e < E; ++e) { c[e] = lc[e]; a[e] = la[e]; }
        load_entries(k + 2, lc, la);
        gather(k + 1, c, x);
        do {                                               // one step, unless more than W rows end in this block
            step_rows();
            step_sums(pr);                                 // (its first LDS fence also frees the product buffer)
        } while (capped);
    }

    store_pending();                                       // the last step's rows
    // the row still open at the end of my chunk is finished by another wave
    bool any = false;
#pragma unroll
    for (int i = 0; i < V; ++i) any |= carry[i] != 0.0f;
    if constexpr (AXPBY) {
#pragma unroll
        for (int i = 0; i < V; ++i) carry[i] *= sc.alpha;
    }
    if (any && lane == 0 && is < M) add_to_row(Y + (size_t)is * ldy + n0, carry);
    }   // next chunk
}

// ===========================================================================
// nnz-balanced, sequential reduction with LDS-staged tiles (Sections 2.1.3, 1)
// ===========================================================================
//
// A wave stages a tile of W = 512 merge-path items in LDS: its entries
// (colidx, val) with coalesced loads (coalesced sparse-row caching) and the
// end offsets of the rows that end in it.  Its 64/G lane groups then each walk
// one run of U = W*G/64 consecutive items in order; lane gl of a group owns V
// dense columns, so per entry a group reads one contiguous piece of a row of
// X.  At a row end the accumulator is flushed.  A row whose items all lie in
// the run is stored directly (empty rows flush a zero accumulator, which is
// how they get their zeros).  A row that crosses run boundaries inside the
// tile is summed in LDS: every run adds its part to the slot named after the
// run the row started in, and after the walk one group writes the slot out -
// with a plain store if the row also ended inside the tile.  Only rows that
// cross the tile's own ends go to memory with atomic adds (prepare kernel:
// rows split by a tile boundary).
// blockIdx.y selects the block of G*V dense columns.

constexpr int kNbSrTile = 512;
constexpr int kNbSrLogTile = 9;

template <int V, bool XBUF, int DEPTH, bool AXPBY = false, bool RAGGED = false>
__global__ __launch_bounds__(kBlock) void nb_sr_kernel(int M, long long K, int N, int ldx, int ldy, const int* __restrict__ rowptr,
                                                        const int* __restrict__ colidx,
                                                        const float* __restrict__ vals,
                                                        const float* __restrict__ X, float* __restrict__ Y,
                                                        int logG, int cols_per_block, Scaling sc = Scaling{1.0f, 0.0f},
                                                        unsigned pinned_blocks = 0) {
    constexpr int W = kNbSrTile;
    constexpr int kStoreAux = V == 4 ? 2 : 0;           // results leave non-temporal when rows are 16 bytes or more per lane
    constexpr int kSlotFloats = 2 * kWave * V;          // (64/G + 1) slots of G*V floats each, G <= 64
    __shared__ __align__(16) int s_col[kWavesPerBlock][W];
    __shared__ __align__(16) float s_val[kWavesPerBlock][W];
    __shared__ __align__(16) unsigned short s_end[kWavesPerBlock][W + 8];   // end offsets (minus js) of the rows ending in the tile
    __shared__ __align__(16) float s_slot[kWavesPerBlock][kSlotFloats];     // slots are read 4 * V bytes at a time
    __shared__ int s_slot_row[kWavesPerBlock][kWave + 4];   // row of each slot (-1: unused)
    __shared__ int s_slot_end[kWavesPerBlock][kWave + 4];   // 1: the slot's row ended inside the tile
    const int lane = lane_id();
    const int wib = wave_in_block();
    int* cc = s_col[wib];
    float* cv = s_val[wib];
    unsigned short* ends = s_end[wib];
    float* slot_acc = s_slot[wib];
    int* slot_row = s_slot_row[wib];
    int* slot_end = s_slot_end[wib];

    const int G = 1 << logG;
    const int gl = lane & (G - 1);
    const int g = lane >> logG;
    const int groups = kWave >> logG;
    const int logU = kNbSrLogTile - 6 + logG;
    const unsigned U = 1u << logU;
    // Column block and place in the chunk list.  Normally blockIdx.y is the column block and blockIdx.x (made
    // XCD-contiguous) the place.  pinned_blocks = nb > 0 (nb in {2, 4}, or 8 for a comparison; gridDim = (8 k, 1)): the
    // workgroups of XCD x all take column block x % nb, so that an L2 only ever sees one block's slice of X; the
    // 8 / nb XCDs of a block share its chunk list, each a contiguous part.
    unsigned col_block = blockIdx.y;
    unsigned wg = 0, nwg = 0;
    if (pinned_blocks) {
        const unsigned x = blockIdx.x % kXcd, i = blockIdx.x / kXcd, per_xcd = gridDim.x / kXcd;
        col_block = x % pinned_blocks;
        wg = (x / pinned_blocks) * per_xcd + i;
        nwg = (kXcd / pinned_blocks) * per_xcd;
    }
    const LaneColumns mine = lane_columns<V, RAGGED>(col_block, cols_per_block, gl, N);
    const long long n = mine.first;
    const bool col_ok = mine.any;
    const int tail = N % V;                  // columns of the lane that shares its window (RAGGED)

    // chunks start at multiples of U: runs stay aligned
    const ChunkPlan plan = pinned_blocks ? plan_chunks(rowptr, M, (unsigned)logU, wg, nwg) : plan_chunks(rowptr, M, (unsigned)logU);
    const unsigned nnz = plan.nnz;
    const unsigned long long y_elems = dense_bytes(M, ldy, N) / 4ull;
    // XBUF: the dense operand is read through a descriptor (its byte offsets fit 32 bits)
    const unsigned long long x_bytes = dense_bytes(K, ldx, N);
    const __amdgpu_buffer_rsrc_t rx = make_buffer(X, XBUF ? x_bytes : 0ull);
    const unsigned n_bytes = (unsigned)n * 4u;

    for (unsigned sub = 0; sub < kSubRanges; ++sub) {
    unsigned d0, d1;
    if (!plan.range(sub, d0, d1)) continue;
    int is = wave_merge_rows_before(rowptr, M, d0, lane);
    unsigned js = d0 - (unsigned)is;
    for (unsigned ds = d0; ds < d1; ds += W) {
        const unsigned de = (d1 - ds > (unsigned)W) ? ds + W : d1;

        wave_lds_sync();                        // previous tile's readers are done
        // entries: at most W, the exact count follows from the row ends
        {
            const unsigned long long bytes = (unsigned long long)(nnz - js) * 4ull;
            const __amdgpu_buffer_rsrc_t rc = make_buffer(colidx + js, bytes);
            const __amdgpu_buffer_rsrc_t ra = make_buffer(vals + js, bytes);
#pragma unroll
            for (int k = 0; k < W / kWave; ++k) {
                const int e = k * kWave + lane;
                cc[e] = buffer_stream_i32(rc, (unsigned)e * 4u);
                cv[e] = buffer_stream_f32(ra, (unsigned)e * 4u);
            }
        }
        // slots for the rows that cross run boundaries inside the tile
#pragma unroll
        for (int k = 0; k < kSlotFloats / kWave; ++k) slot_acc[k * kWave + lane] = 0.0f;
        slot_row[lane] = -1; slot_end[lane] = 0;
        if (lane == 0) { slot_row[kWave] = -1; slot_end[kWave] = 0; }
        // end offsets of rows is, is+1, ... while their end marker is inside the tile: 64 candidates first,
        // and if all of them end here (a tile crowded with short or empty rows) the other 448 in one go
        int ie = is;
        {
            const unsigned long long rbytes = is < M ? (unsigned long long)(M + 1 - is) * 4ull : 0ull;
            const __amdgpu_buffer_rsrc_t rr = make_buffer(rowptr + is, rbytes);     // rows past the last read as 0
            auto take = [&](int m, unsigned e) {
                const long long r = (long long)is + m * kWave + lane;
                const bool in = r < M && (unsigned)r + e < de;
                if (in) ends[m * kWave + lane] = (unsigned short)(e - js);
                return (int)__popcll(__ballot(in));
            };
            int cnt = take(0, (unsigned)__builtin_amdgcn_raw_buffer_load_b32(rr, (unsigned)(lane + 1) * 4u, 0, 0));
            ie += cnt;
            if (cnt == kWave) {
                unsigned e[W / kWave - 1];
#pragma unroll
                for (int m = 1; m < W / kWave; ++m)
                    e[m - 1] = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(rr, (unsigned)(m * kWave + lane + 1) * 4u, 0, 0);
#pragma unroll
                for (int m = 1; m < W / kWave; ++m) {
                    if (cnt == kWave) { cnt = take(m, e[m - 1]); ie += cnt; }
                }
            }
        }
        const int nrows = ie - is;              // rows ending in this tile
        const unsigned rs_first = is < M ? (unsigned)rowptr[is] : nnz;   // start offset of row `is`
        wave_lds_sync();

        // rows [is, ie) end in this tile; their results leave through one descriptor based at row `is`
        const unsigned long long first_elem = (unsigned long long)is * (unsigned)ldy;
        const unsigned long long left = first_elem < y_elems ? (y_elems - first_elem) * 4ull : 0ull;
        const __amdgpu_buffer_rsrc_t yrows = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(Y + first_elem), 0, left > 0xffffffffull ? 0xffffffffu : (unsigned)left, kBufferFlags);

        // rows without entries get their zeros here, all groups together (group g: local rows g, g + groups, ...),
        // so that the walk below meets a store only where a row with entries ends.  With four columns per lane
        // results are stored non-temporal here and in the walk: nobody reads them again, the L2 is for rows of X
        // (1-4 % measured at N >= 8; at N = 1, 2 the narrow stores were 4-8 % slower that way).
        {
            float zero[V];
#pragma unroll
            for (int i = 0; i < V; ++i) zero[i] = 0.0f;
            for (int t0 = 0; t0 < nrows; t0 += 4 * groups) {      // wave-uniform; four independent stores per round
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int tz = t0 + q * groups + g;
                    bool empty = false;
                    if (tz < nrows) {
                        const int end = (int)ends[tz];
                        const int start = tz == 0 ? (int)(rs_first - js) : (int)ends[tz - 1];   // negative: began before the tile
                        empty = end == start;
                    }
                    const unsigned off = (empty && col_ok) ? (unsigned)tz * (unsigned)ldy * 4u + n_bytes : kOutOfRange;
                    if constexpr (AXPBY) {
                        float out[V];
#pragma unroll
                        for (int i = 0; i < V; ++i) out[i] = 0.0f;
                        scale_into<V>(out, yrows, off, sc);               // beta * Y
                        buffer_store_columns<V, RAGGED, kStoreAux, true>(yrows, off, out, mine.skip, tail);
                    } else {
                        buffer_store_columns<V, RAGGED, kStoreAux, false>(yrows, off, zero, mine.skip, tail);
                    }
                }
            }
        }

        // first local row in [lo, hi) whose end offset lies beyond `off` (end offsets never decrease); hi if none
        auto first_row_ending_after = [&](int lo, int hi, unsigned off) {
            if (lo >= hi || js + ends[lo] > off) return lo;          // the usual case: the next row has entries
            ++lo;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (js + ends[mid] <= off) lo = mid + 1; else hi = mid;
            }
            return lo;
        };

        // ---- my run: diagonals [dg, dh) = entries [j, j_end) and the end markers of rows [t, t_end)
        const unsigned dg = ds + ((unsigned)g << logU);
        const bool has_run = dg < de && col_ok;
        int t = 0, t_end = 0;
        unsigned j = 0, j_end = 0, next_end = kNoRow, cur_first = 0;
        if (has_run) {
            const unsigned dh = (de - dg > U) ? dg + U : de;
            // rows (local index t, row is+t) whose end marker lies before a diagonal d: is+t + ends[t] < d
            auto rows_before = [&](unsigned d) {
                int lo = 0, hi = nrows;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if ((unsigned)(is + mid) + js + ends[mid] < d) lo = mid + 1; else hi = mid;
                }
                return lo;
            };
            t = rows_before(dg);                             // first row (local) to end at or after dg
            t_end = rows_before(dh);                         // rows [t, t_end) end inside my run
            j = dg - (unsigned)(is + t);                     // first entry of my run
            j_end = dh - (unsigned)(is + t_end);
            // rows without entries at the head of the run are done already
            const unsigned start_off = t == 0 ? rs_first : js + ends[t - 1];   // where row t's entries begin
            t = first_row_ending_after(t, t_end, start_off);
            next_end = t < nrows ? js + ends[t] : kNoRow;    // end offset of the current row
            cur_first = (unsigned)(is + t) + start_off;      // first item of the current row
        }
        // lanes without a run keep j == j_end and t == t_end: they issue the same instructions, switched off

        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.0f;

        // a partial sum of row is+t (it crosses my run's ends) goes to the slot of the run it started in
        auto to_slot = [&](bool ended) {
            const int s = cur_first < ds ? 0 : (int)((cur_first - ds) >> logU) + 1;
            float* dst = slot_acc + (size_t)(s * G + gl) * V;
#pragma unroll
            for (int i = 0; i < V; ++i) atomicAdd(dst + i, acc[i]);
            if (gl == 0) { slot_row[s] = is + t; if (ended) slot_end[s] = 1; }   // every writer of slot_row[s] writes the same row
        };
        // The current row ends here (closing: its end marker lies in my run).  A row that began inside my run is
        // stored, one that began earlier goes to its slot.  The store is issued by the whole wave whenever any
        // group closes a row - switched off where none does - so no memory operation sits in a divergent branch.
        auto close_row = [&](bool closing) {
            if (__ballot(closing) != 0ull) {                 // wave-uniform
                const bool direct = closing && cur_first >= dg;
                const unsigned off = direct ? (unsigned)t * (unsigned)ldy * 4u + n_bytes : kOutOfRange;
                if constexpr (AXPBY) {
                    float out[V];
#pragma unroll
                    for (int i = 0; i < V; ++i) out[i] = acc[i];
                    scale_into<V>(out, yrows, off, sc);
                    buffer_store_columns<V, RAGGED, kStoreAux, true>(yrows, off, out, mine.skip, tail);
                } else {
                    buffer_store_columns<V, RAGGED, kStoreAux, false>(yrows, off, acc, mine.skip, tail);
                }
                if (closing) {
                    if (!direct) to_slot(true);
#pragma unroll
                    for (int i = 0; i < V; ++i) acc[i] = 0.0f;
                    const unsigned off = next_end;           // the next row's entries begin where this one's end
                    t = first_row_ending_after(t + 1, t_end, off);   // rows without entries: zeros written above
                    cur_first = (unsigned)(is + t) + off;
                    next_end = t < nrows ? js + ends[t] : kNoRow;
                }
            }
        };
        // the dense-row load of entry p into register set u; switched off past the run's last entry
        float x[DEPTH][V]; float a[DEPTH];
        auto issue = [&](int u, unsigned p) {
            const bool ok = p < j_end;
            const int e = ok ? (int)(p - js) : 0;
            a[u] = ok ? cv[e] : 0.0f;
            const unsigned c = (unsigned)cc[e];
            if constexpr (XBUF) {
                buffer_load_vec<V>(rx, ok ? c * (unsigned)ldx * 4u + n_bytes : kOutOfRange, x[u]);
            } else {
                load_vec_dword_aligned<V>(X + (size_t)(ok ? c : 0u) * ldx + (col_ok ? n : 0), x[u]);
#pragma unroll
                for (int i = 0; i < V; ++i) x[u][i] = ok ? x[u][i] : 0.0f;
            }
        };
        // DEPTH loads stay in flight: entry p is consumed while entry p + DEPTH is requested
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) issue(u, j + u);
        for (unsigned p0 = j; __ballot(p0 < j_end) != 0ull; p0 += DEPTH) {     // the same trip count for every lane
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const unsigned p = p0 + u;
                close_row(p < j_end && next_end == p);       // the row before entry p is complete
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] = fmaf(a[u], x[u][i], acc[i]);   // a is 0 past the end
                issue(u, p + DEPTH);
            }
        }
        close_row(t < t_end);                                // the row whose end marker follows my last entry
        // what is left belongs to a row that goes on after my run (if the run held entries of it)
        if (has_run && (unsigned)(is + t) + j_end > cur_first) to_slot(false);
        wave_lds_sync();                                     // every run has added its parts

        // one group per slot writes the rows that crossed run boundaries: slot g+1 by group g, slot 0 by group 0 too
        if (col_ok) {
            for (int s = (g == 0 ? 0 : g + 1); s <= g + 1 && s <= groups; ++s) {
                const int row = slot_row[s];
                if (row >= 0) {
                    float val[V];
                    load_vec<V>(slot_acc + (size_t)(s * G + gl) * V, val);
                    float* y = Y + (size_t)row * ldy + n;
                    // started inside the tile (s > 0) and ended inside it: nobody else has a part of this row
                    const bool whole = s > 0 && slot_end[s];
                    if constexpr (AXPBY) {
                        if (whole) {
                            scale_into<V, true>(val, y, sc);
                        } else {
#pragma unroll
                            for (int i = 0; i < V; ++i) val[i] *= sc.alpha;          // lands on beta * Y (prepare)
                        }
                    }
                    if (RAGGED && mine.skip != 0) {
#pragma unroll
                        for (int i = 1; i < V; ++i) {
                            if (i >= mine.skip) { if (whole) y[i] = val[i]; else unsafeAtomicAdd(y + i, val[i]); }
                        }
                    } else if (whole) {
                        store_vec_dword_aligned<V>(y, val);
                    } else {
                        atomic_add_vec<V>(y, val);
                    }
                }
            }
        }

        js = de - (unsigned)ie;
        is = ie;
    }
    }   // next chunk
}

// ===========================================================================
// row statistics of a matrix that lives in device memory (the selector's metrics, Section 2.2)
// ===========================================================================
// ws[0] sum of len^2, [1] max len, [2] min len, [3] non-empty rows whose span was taken,
// [4] sum of (largest - smallest column + 1), [5] a row pointer decreased, [6] rowptr[0], [7] rowptr[M].
// All integer, so the result does not depend on the order in which waves arrive.
constexpr int kFeatureWords = 8;
constexpr int kFeatureLongRow = 128;   // longer rows are scanned by the whole wave

__global__ void features_init_kernel(unsigned long long* __restrict__ ws) {
    if (blockIdx.x == 0 && threadIdx.x < kFeatureWords) ws[threadIdx.x] = threadIdx.x == 2 ? ~0ull : 0ull;
}

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int mask) {
    const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)v, mask, kWave);
    const unsigned hi = (unsigned)__shfl_xor((int)(unsigned)(v >> 32), mask, kWave);
    return ((unsigned long long)hi << 32) | lo;
}

__global__ __launch_bounds__(kBlock) void features_kernel(int M, const int* __restrict__ rowptr,
                                                           const int* __restrict__ colidx,
                                                           unsigned long long* __restrict__ ws) {
    const int lane = lane_id();
    const long long nwaves = (long long)gridDim.x * kWavesPerBlock;
    const long long gw = (long long)blockIdx.x * kWavesPerBlock + wave_in_block();
    unsigned long long sq = 0, mx = 0, mn = ~0ull, rows = 0, span = 0, bad = 0;
    for (long long r0 = gw * kWave; r0 < M; r0 += nwaves * kWave) {
        const long long row = r0 + lane;
        const bool live = row < M;
        int s = 0, e = 0;
        if (live) { s = rowptr[row]; e = rowptr[row + 1]; }
        long long len = (long long)e - (long long)s;
        if (len < 0) { bad = 1; len = 0; }
        if (live) {
            const unsigned long long l = (unsigned long long)len;
            sq += l * l;
            mx = l > mx ? l : mx;
            mn = l < mn ? l : mn;
        }
        if (colidx != nullptr) {
            const bool long_row = live && len > kFeatureLongRow;
            if (live && len > 0 && !long_row) {
                int lo = colidx[s], hi = lo;
                for (int p = s + 1; p < e; ++p) {
                    const int c = colidx[p];
                    lo = c < lo ? c : lo;
                    hi = c > hi ? c : hi;
                }
                span += (unsigned long long)((long long)hi - lo + 1);
                rows += 1;
            }
            unsigned long long todo = __ballot(long_row);
            while (todo) {                                   // wave-uniform
                const int src = __ffsll((long long)todo) - 1;
                todo &= todo - 1;
                const int ss = __shfl(s, src, kWave), ee = __shfl(e, src, kWave);
                int lo = 0x7fffffff, hi = -0x7fffffff - 1;
                for (int p = ss + lane; p < ee; p += kWave) {
                    const int c = colidx[p];
                    lo = c < lo ? c : lo;
                    hi = c > hi ? c : hi;
                }
#pragma unroll
                for (int m = 1; m < kWave; m <<= 1) {
                    const int ol = __shfl_xor(lo, m, kWave), oh = __shfl_xor(hi, m, kWave);
                    lo = ol < lo ? ol : lo;
                    hi = oh > hi ? oh : hi;
                }
                if (lane == src) {
                    span += (unsigned long long)((long long)hi - lo + 1);
                    rows += 1;
                }
            }
        }
    }
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        sq += shfl_xor_u64(sq, m);
        rows += shfl_xor_u64(rows, m);
        span += shfl_xor_u64(span, m);
        bad |= shfl_xor_u64(bad, m);
        const unsigned long long omx = shfl_xor_u64(mx, m), omn = shfl_xor_u64(mn, m);
        mx = omx > mx ? omx : mx;
        mn = omn < mn ? omn : mn;
    }
    if (lane == 0) {
        atomicAdd(&ws[0], sq);
        atomicMax(&ws[1], mx);
        atomicMin(&ws[2], mn);
        if (rows) atomicAdd(&ws[3], rows);
        if (span) atomicAdd(&ws[4], span);
        if (bad) atomicMax(&ws[5], 1ull);
        if (gw == 0) {
            ws[6] = (unsigned long long)(long long)rowptr[0];
            ws[7] = (unsigned long long)(long long)rowptr[M];
        }
    }
}

// ===========================================================================
// 64-bit row pointers: slabs of rows whose entry positions fit 32 bits
// ===========================================================================
// The kernels address entries with 32-bit positions.  A matrix with more than 2^31 stored entries is cut into
// slabs of consecutive rows: slab k starts at the first row whose pointer reaches k * slab_entries.  One thread
// per cut: out[2k] = the row, out[2k+1] = its pointer (the slab's base); cut nslabs is (M, rowptr[M]).
__global__ void i64_slab_bounds_kernel(long long M, const long long* __restrict__ rowptr, int nslabs, long long slab_entries,
                                       long long* __restrict__ out) {
    const int k = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (k > nslabs) return;
    long long r = M;
    if (k < nslabs) {
        const long long target = (long long)k * slab_entries;
        long long lo = 0, hi = M;                       // first r in [0, M] with rowptr[r] >= target
        while (lo < hi) {
            const long long mid = lo + (hi - lo) / 2;
            if (rowptr[mid] < target) lo = mid + 1; else hi = mid;
        }
        r = lo;
    }
    out[2 * k] = r;
    out[2 * k + 1] = rowptr[r];
}

// The 32-bit row pointers of one slab: out[i] = rowptr[first + i] - base for i in [0, rows].
__global__ __launch_bounds__(kBlock) void i64_slab_rowptr_kernel(long long rows, const long long* __restrict__ rowptr_first,
                                                                  long long base, int* __restrict__ out) {
    const long long nthreads = (long long)gridDim.x * kBlock;
    for (long long i = (long long)blockIdx.x * kBlock + threadIdx.x; i <= rows; i += nthreads)
        out[i] = (int)(rowptr_first[i] - base);
}

// ===========================================================================
// measurement aids: pure gather, the memory side of the parallel and of the sequential kernels, plain streaming copy
// ===========================================================================

// Streams idx and gathers x[idx[i]], four independent gathers in flight per
// lane; nothing else.  One partial sum per thread keeps the loads alive.
__global__ __launch_bounds__(kBlock) void gather_probe_kernel(float* __restrict__ out, const float* __restrict__ x,
                                                               const int* __restrict__ idx, long long n) {
    const long long nthreads = (long long)gridDim.x * kBlock;
    const long long t = (long long)blockIdx.x * kBlock + threadIdx.x;
    float acc = 0.0f;
    for (long long base = t; base < n; base += nthreads * 4) {
        int c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long long i = base + u * nthreads;
            c[u] = i < n ? stream_load(idx + i) : -1;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc += c[u] >= 0 ? x[c[u]] : 0.0f;
    }
    out[t] = acc;
}

// Floor of the parallel-reduction kernels: what they do to memory and nothing else.  A wave takes blocks of
// 512 consecutive entries; lane l loads entries 64 e + l (coalesced, non-temporal), gathers V dense values for
// each with one vector load and multiplies-adds them into V private sums.  The pipeline is the entry-block
// kernel's: while block b is multiplied, the gathers of block b + 1 and the entries of block b + 2 are in
// flight; arriving entries wait in a second register set and are moved over once block b is done.  No row
// bounds, no reduction across lanes, no result rows: the per-lane sums go to out[thread * V + i] so that the
// loads stay alive (and so that a test can check their total).
template <int V>
__global__ __launch_bounds__(kBlock) void stream_gather_fma_probe_kernel(float* __restrict__ out, const float* __restrict__ X,
                                                                         long long K, int ldx, const int* __restrict__ colidx,
                                                                         const float* __restrict__ vals, long long nnz) {
    constexpr int E = 8;
    constexpr long long W = kWave * E;
    const int lane = lane_id();
    const long long nwaves = (long long)gridDim.x * kWavesPerBlock;
    const long long gw = (long long)xcd_contiguous(blockIdx.x, gridDim.x) * kWavesPerBlock + wave_in_block();
    const long long nblocks = (nnz + W - 1) / W;
    const long long b0 = nblocks * gw / nwaves, b1 = nblocks * (gw + 1) / nwaves;      // my contiguous share
    const unsigned long long x_bytes = dense_bytes(K, ldx, V);
    const bool x_small = x_bytes <= 0xffffffffull;
    const __amdgpu_buffer_rsrc_t rx = make_buffer(X, x_small ? x_bytes : 0ull);
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.0f;
    int c[E], lc[E];
    float a[E], la[E], x[E][V];
    // entries of block b into the arriving set (nothing past my share or past the arrays' end: zeros, which add nothing)
    auto load_entries = [&](long long b) {
        const long long from = b * W;
        const unsigned long long bytes = (b < b1 && from < nnz) ? (unsigned long long)(nnz - from) * 4ull : 0ull;
        const __amdgpu_buffer_rsrc_t rc = make_buffer(colidx + (bytes ? from : 0), bytes);
        const __amdgpu_buffer_rsrc_t ra = make_buffer(vals + (bytes ? from : 0), bytes);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const unsigned off = (unsigned)(e * kWave + lane) * 4u;
            lc[e] = buffer_stream_i32(rc, off);
            la[e] = buffer_stream_f32(ra, off);
        }
    };
    auto take_entries = [&]() {
#pragma unroll
        for (int e = 0; e < E; ++e) { c[e] = lc[e]; a[e] = la[e]; }
    };
    // dense values for the entries in c (those of block b)
    auto gather = [&](long long b) {
        const long long left = b < b1 ? nnz - b * W : 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const bool ok = e * kWave + lane < left;
            if (x_small) {
                buffer_load_vec<V>(rx, ok ? (unsigned)c[e] * (unsigned)ldx * 4u : kOutOfRange, x[e]);
            } else {
                load_vec_dword_aligned<V>(X + (size_t)(ok ? c[e] : 0) * ldx, x[e]);
            }
        }
    };
    load_entries(b0);
    take_entries();
    load_entries(b0 + 1);
    gather(b0);
    for (long long b = b0; b < b1; ++b) {
#pragma unroll
        for (int e = 0; e < E; ++e)
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = fmaf(a[e], x[e][i], acc[i]);
        take_entries();
        load_entries(b + 2);
        gather(b + 1);
    }
    const long long t = (long long)blockIdx.x * kBlock + threadIdx.x;
#pragma unroll
    for (int i = 0; i < V; ++i) out[t * V + i] = acc[i];
}

// Floor of the sequential-reduction kernels at width N: a wave stages 512 consecutive entries in LDS with
// coalesced loads, then each of its 64 / G lane groups walks 512 G / 64 of them in order, one dwordx4 load of the
// entry's row of X per lane and step (lane gl owns columns [block * 4 G + 4 gl, + 4)), multiply-add into four private
// sums.  No rows, no stores inside the walk.  blockIdx.y selects the block of 4 G columns.  N must be a multiple of 4.
__global__ __launch_bounds__(kBlock) void row_gather_probe_kernel(float* __restrict__ out, const float* __restrict__ X,
                                                                  long long K, int N, int ldx, const int* __restrict__ colidx,
                                                                  const float* __restrict__ vals, long long nnz, int logG) {
    constexpr int W = 512;
    __shared__ __align__(16) int s_col[kWavesPerBlock][W];
    __shared__ __align__(16) float s_val[kWavesPerBlock][W];
    const int lane = lane_id();
    const int wib = wave_in_block();
    int* cc = s_col[wib];
    float* cv = s_val[wib];
    const int G = 1 << logG;
    const int gl = lane & (G - 1), g = lane >> logG;
    const int U = W >> (6 - logG);                                   // entries per group and tile
    const long long n = (long long)blockIdx.y * 4 * G + 4 * gl;      // my first column
    const bool col_ok = n + 4 <= N;
    const long long nwaves = (long long)gridDim.x * kWavesPerBlock;
    const long long gw = (long long)xcd_contiguous(blockIdx.x, gridDim.x) * kWavesPerBlock + wib;
    const long long ntiles = (nnz + W - 1) / W;
    const long long t0 = ntiles * gw / nwaves, t1 = ntiles * (gw + 1) / nwaves;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (long long t = t0; t < t1; ++t) {
        const long long from = t * W;
        const __amdgpu_buffer_rsrc_t rc = make_buffer(colidx + from, (unsigned long long)(nnz - from) * 4ull);
        const __amdgpu_buffer_rsrc_t ra = make_buffer(vals + from, (unsigned long long)(nnz - from) * 4ull);
        wave_lds_sync();
#pragma unroll
        for (int k = 0; k < W / kWave; ++k) {
            const int e = k * kWave + lane;
            cc[e] = buffer_stream_i32(rc, (unsigned)e * 4u);      // past the end: column 0, value 0
            cv[e] = buffer_stream_f32(ra, (unsigned)e * 4u);
        }
        wave_lds_sync();
        if (col_ok) {
            for (int e = g * U; e < (g + 1) * U; ++e) {
                float x[4];
                load_vec_dword_aligned<4>(X + (size_t)cc[e] * ldx + n, x);
                const float a = cv[e];
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] = fmaf(a, x[i], acc[i]);
            }
        }
    }
    const long long th = ((long long)blockIdx.y * gridDim.x + blockIdx.x) * kBlock + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) out[th * 4 + i] = acc[i];
}

__global__ __launch_bounds__(kBlock) void copy_kernel(float* __restrict__ dst, const float* __restrict__ src,
                                                       long long n) {
    const long long nthreads = (long long)gridDim.x * kBlock;
    const long long t = (long long)blockIdx.x * kBlock + threadIdx.x;
    const long long n4 = n / 4;
    const float4* s4 = reinterpret_cast<const float4*>(src);
    float4* d4 = reinterpret_cast<float4*>(dst);
    for (long long i = t; i < n4; i += nthreads) d4[i] = s4[i];
    for (long long i = n4 * 4 + t; i < n; i += nthreads) dst[i] = src[i];
}

}  // namespace dgsp
