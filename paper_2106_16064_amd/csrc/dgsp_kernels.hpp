// The four CSR SpMV/SpMM kernels of the paper's design space (Section 2.1):
// {row-split, nnz-balanced} x {sequential, parallel reduction}, for gfx950.
//
// Common shape of all four
//   * 256-thread workgroups = 4 waves; every cooperative step is wave-local
//     (DPP moves or wave-private LDS), so there is no s_barrier anywhere.
//   * `V` (1, 2 or 4) is the vector width of dense-row accesses: one
//     dword / dwordx2 / dwordx4 per lane (vector-type dense-row loading,
//     Section 2.1.2).  The host picks the widest V that divides N and matches
//     the alignment of X and Y.
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
// For N > V the columns are processed V at a time.

__host__ __device__ __forceinline__ int pr_lanes_log2(long long nnz, long long M) {
    // lanes per row ~ average row length, rounded up to a power of two in [2, 64]
    const double avg = M > 0 ? (double)nnz / (double)M : 0.0;
    int lg = 1;
    while (lg < 6 && (double)(1 << lg) < avg) ++lg;
    return lg;
}

template <int V>
__global__ __launch_bounds__(kBlock) void rs_pr_kernel(int M, int N, const int* __restrict__ rowptr,
                                                        const int* __restrict__ colidx,
                                                        const float* __restrict__ vals,
                                                        const float* __restrict__ X, float* __restrict__ Y,
                                                        int logG_in) {
    const int lane = lane_id();
    const int logG = logG_in >= 0 ? logG_in : pr_lanes_log2(rowptr[M], M);
    const int G = 1 << logG;
    const int gl = lane & (G - 1);              // lane inside the group
    const int rows_per_wave = kWave >> logG;
    const unsigned nwaves = gridDim.x * kWavesPerBlock;
    const unsigned gw = xcd_contiguous(blockIdx.x, gridDim.x) * kWavesPerBlock + wave_in_block();
    const unsigned ngroups = ((unsigned)M + rows_per_wave - 1) / rows_per_wave;   // row groups of one wave each

    // XCD-contiguous and interleaved: wave gw of the nwaves takes row groups
    // q*nwaves + gw.  Consecutive waves (same block, same XCD) take consecutive rows.
    for (unsigned rg = gw; rg < ngroups; rg += nwaves) {
        const long long row = (long long)rg * rows_per_wave + (lane >> logG);
        const bool live = row < M;
        unsigned rs = 0, re = 0;
        if (live) { rs = (unsigned)rowptr[row]; re = (unsigned)rowptr[row + 1]; }
        for (int n0 = 0; n0 < N; n0 += V) {
            float acc[V];
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = 0.0f;
            // four independent gathers in flight per lane
            for (unsigned p = rs + gl; p < re; p += 4u * G) {
                int c[4]; float a[4]; float x[4][V];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned q = p + (unsigned)u * G;
                    const bool ok = q < re;
                    c[u] = ok ? colidx[q] : -1;
                    a[u] = ok ? vals[q] : 0.0f;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (c[u] >= 0) load_vec<V>(X + (size_t)c[u] * N + n0, x[u]);
                    else {
#pragma unroll
                        for (int i = 0; i < V; ++i) x[u][i] = 0.0f;
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int i = 0; i < V; ++i) acc[i] = fmaf(a[u], x[u][i], acc[i]);
            }
            segmented_scan<V>(acc, gl, lane, G);   // all 64 lanes arrive here together
            if (live && gl == G - 1) store_vec<V>(Y + (size_t)row * N + n0, acc);
        }
    }
}

// ===========================================================================
// Row-split, sequential reduction with coalesced sparse-row caching
// (Section 2.1.3)
// ===========================================================================
//
// 2^logG lanes own a row and V*2^logG dense columns (lane gl owns columns
// [cb*G*V + gl*V, +V)).  The group loads a slice of the row's (colidx, val)
// pairs with coalesced loads, parks it in its private LDS slot, then every
// lane walks the cached pairs and accumulates its own columns: the dense
// accesses of a group are one contiguous 4*V*G-byte piece of a row of X.
// blockIdx.y selects the column block when N > 64*V.

constexpr int kRsSrSlot = 512;   // cached pairs per wave

template <int V>
__global__ __launch_bounds__(kBlock) void rs_sr_kernel(int M, int N, const int* __restrict__ rowptr,
                                                        const int* __restrict__ colidx,
                                                        const float* __restrict__ vals,
                                                        const float* __restrict__ X, float* __restrict__ Y,
                                                        int logG) {
    __shared__ int s_col[kWavesPerBlock][kRsSrSlot];
    __shared__ float s_val[kWavesPerBlock][kRsSrSlot];
    const int lane = lane_id();
    const int wib = wave_in_block();
    const int G = 1 << logG;
    const int gl = lane & (G - 1);
    const int g = lane >> logG;
    const int rows_per_wave = kWave >> logG;
    const int S = G >= 8 ? G : 8;               // pairs cached per group and round
    const int R = S >> logG;                    // loads per lane and round
    int* cc = s_col[wib] + g * S;
    float* cv = s_val[wib] + g * S;

    const long long n = ((long long)blockIdx.y * G + gl) * V;   // my first dense column
    const bool col_ok = n < N;

    const unsigned nwaves = gridDim.x * kWavesPerBlock;
    const unsigned gw = xcd_contiguous(blockIdx.x, gridDim.x) * kWavesPerBlock + wib;
    const unsigned ngroups = ((unsigned)M + rows_per_wave - 1) / rows_per_wave;

    for (unsigned rg = gw; rg < ngroups; rg += nwaves) {
        const long long row = (long long)rg * rows_per_wave + g;
        const bool live = row < M;
        unsigned rs = 0, re = 0;
        if (live) { rs = (unsigned)rowptr[row]; re = (unsigned)rowptr[row + 1]; }
        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.0f;

        for (unsigned base = rs; base < re; base += (unsigned)S) {
            wave_lds_sync();                    // last round's readers are done
            for (int i = 0; i < R; ++i) {
                const int e = i * G + gl;
                const unsigned p = base + (unsigned)e;
                if (p < re) { cc[e] = stream_load(colidx + p); cv[e] = stream_load(vals + p); }
            }
            wave_lds_sync();
            const int cnt = (re - base) < (unsigned)S ? (int)(re - base) : S;
            if (col_ok) {
                for (int j = 0; j < cnt; j += 4) {
                    float x[4][V]; float a[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        if (j + u < cnt) {
                            const int c = cc[j + u];
                            a[u] = cv[j + u];
                            load_vec<V>(X + (size_t)c * N + n, x[u]);
                        } else {
                            a[u] = 0.0f;
#pragma unroll
                            for (int i = 0; i < V; ++i) x[u][i] = 0.0f;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int i = 0; i < V; ++i) acc[i] = fmaf(a[u], x[u][i], acc[i]);
                }
            }
        }
        if (live && col_ok) store_vec<V>(Y + (size_t)row * N + n, acc);
    }
}

// ===========================================================================
// nnz-balanced kernels: common partition
// ===========================================================================
//
// The stored entries [0, nnz) are cut into tiles of T consecutive entries; the
// tiles are dealt to the waves of the grid in contiguous ranges (wave w owns
// tiles [w*tpw, (w+1)*tpw)), XCD-contiguously.  A wave finds the row of its
// first entry once (wave_find_row) and then only walks forward.
//
// Rows that end up split between tiles (or, in the sequential kernel, between
// the runs of different lane groups) are combined with fp32 atomic adds; the
// paper does not say how partial rows of different warps meet.  That needs
// zeros underneath, and rows without entries need zeros too, so a small
// "prepare" kernel runs first: it zeroes exactly the rows that are empty or
// that cross a multiple of the unit U = 2^logU, and nothing else.  Rows that
// lie inside one unit are written once, with a plain store.

__global__ __launch_bounds__(kBlock) void nb_prepare_kernel(int M, int N, const int* __restrict__ rowptr,
                                                             float* __restrict__ Y, int logU, int logP) {
    // 2^logP consecutive threads share a row and stride over its N columns
    const long long t = (long long)blockIdx.x * kBlock + threadIdx.x;
    const long long row = t >> logP;
    if (row >= M) return;
    const unsigned rs = (unsigned)rowptr[row], re = (unsigned)rowptr[row + 1];
    const bool split = (rs == re) || ((rs >> logU) != ((re - 1) >> logU));
    if (!split) return;
    float* y = Y + (size_t)row * N;
    for (int n = (int)(t & ((1 << logP) - 1)); n < N; n += 1 << logP) y[n] = 0.0f;
}

struct TileRange {
    unsigned first, last;   // tiles [first, last)
    unsigned nnz;
};

template <int T>
__device__ __forceinline__ TileRange my_tiles(const int* __restrict__ rowptr, int M) {
    TileRange r;
    r.nnz = (unsigned)rowptr[M];
    const unsigned ntiles = r.nnz / T + (r.nnz % T != 0);
    const unsigned nwaves = gridDim.x * kWavesPerBlock;
    const unsigned gw = xcd_contiguous(blockIdx.x, gridDim.x) * kWavesPerBlock + wave_in_block();
    const unsigned tpw = ntiles / nwaves + (ntiles % nwaves != 0);
    const unsigned long long f = (unsigned long long)gw * tpw;
    r.first = f < ntiles ? (unsigned)f : ntiles;
    r.last = f + tpw < ntiles ? (unsigned)(f + tpw) : ntiles;
    return r;
}

// ===========================================================================
// nnz-balanced, parallel reduction: vectorized segment reduction (Section 2.1.1)
// ===========================================================================
//
// Tile = KCH chunks of 64 entries.  In chunk j lane l holds entry
// ts + 64*j + l (coalesced dword loads), gathers V dense values, multiplies,
// and the chunk is reduced with the segmented DPP scan.  The last lane of a
// segment "dumps" the row's sum (the paper words this as comparing with the
// neighbour lane; here the lane compares its position with its row's end,
// which it knows from the row search).  A row running from chunk j into
// chunk j+1 hands its partial sum over in a register (lane 63 -> lane 0),
// so atomics are needed only where a row crosses the tile.

template <int V, int KCH>
__global__ __launch_bounds__(kBlock) void nb_pr_kernel(int M, int N, const int* __restrict__ rowptr,
                                                        const int* __restrict__ colidx,
                                                        const float* __restrict__ vals,
                                                        const float* __restrict__ X, float* __restrict__ Y) {
    constexpr int T = kWave * KCH;
    constexpr int WMAX = T < 512 ? T : 512;
    __shared__ int s_win[kWavesPerBlock][WMAX];
    const int lane = lane_id();
    int* win = s_win[wave_in_block()];

    const TileRange tr = my_tiles<T>(rowptr, M);
    if (tr.first >= tr.last) return;
    const unsigned nnz = tr.nnz;

    int r_lo = wave_find_row(rowptr, M, tr.first * (unsigned)T, lane);
    unsigned rs_lo = (unsigned)rowptr[r_lo];

    for (unsigned tile = tr.first; tile < tr.last; ++tile) {
        const unsigned ts = tile * (unsigned)T;
        const unsigned te = (nnz - ts > (unsigned)T) ? ts + T : nnz;

        // sparse entries first, so their latency overlaps the row search
        int c[KCH]; float a[KCH];
#pragma unroll
        for (int j = 0; j < KCH; ++j) {
            const unsigned p = ts + j * kWave + lane;
            const bool ok = p < te;
            c[j] = ok ? stream_load(colidx + p) : -1;
            a[j] = ok ? stream_load(vals + p) : 0.0f;
        }

        const RowWindow w = build_row_window<WMAX>(rowptr, M, win, r_lo, rs_lo, te, lane);
        int cnt[KCH]; unsigned rs[KCH], re[KCH];
#pragma unroll
        for (int j = 0; j < KCH; ++j) {
            unsigned p = ts + j * kWave + lane;
            p = p < te ? p : te - 1;
            w.locate(p, cnt[j], rs[j], re[j]);
        }

        for (int n0 = 0; n0 < N; n0 += V) {
            float carry[V];
#pragma unroll
            for (int i = 0; i < V; ++i) carry[i] = 0.0f;
#pragma unroll
            for (int j = 0; j < KCH; ++j) {
                const unsigned cs = ts + j * kWave;           // chunk [cs, ce)
                if (cs >= te) break;                          // wave-uniform
                const unsigned ce = (te - cs > (unsigned)kWave) ? cs + kWave : te;
                const unsigned p = cs + lane;
                const bool ok = p < te;
                float v[V];
                if (ok) {
                    load_vec<V>(X + (size_t)c[j] * N + n0, v);
#pragma unroll
                    for (int i = 0; i < V; ++i) v[i] *= a[j];
                } else {
#pragma unroll
                    for (int i = 0; i < V; ++i) v[i] = 0.0f;
                }
                if (lane == 0) {
#pragma unroll
                    for (int i = 0; i < V; ++i) v[i] += carry[i];
                }
                const unsigned seg_lo = rs[j] > cs ? rs[j] : cs;
                const int h = ok ? (int)(p - seg_lo) : 0;
                segmented_scan<V>(v, h, lane);

                const unsigned seg_hi = re[j] < ce ? re[j] : ce;
                const bool tail = ok && (p + 1 == seg_hi);
                // does the last lane's row go on in the next chunk of this tile?
                const bool cont = (ce < te) && ((unsigned)read_lane((int)re[j], kWave - 1) > ce);
#pragma unroll
                for (int i = 0; i < V; ++i) carry[i] = cont ? read_lane(v[i], kWave - 1) : 0.0f;
                if (tail && !(cont && lane == kWave - 1)) {
                    float* y = Y + (size_t)((long long)r_lo + cnt[j]) * N + n0;
                    if (rs[j] >= ts && re[j] <= te) store_vec<V>(y, v);
                    else atomic_add_vec<V>(y, v);
                }
            }
        }

        // the row holding the tile's last entry is a lower bound for the next tile
        int lc; unsigned lrs, lre;
        w.locate(te - 1, lc, lrs, lre);
        r_lo = uniform(r_lo + lc);
        rs_lo = (unsigned)uniform((int)lrs);
    }
}

// ===========================================================================
// nnz-balanced, sequential reduction with LDS-staged tiles (Sections 2.1.3, 1)
// ===========================================================================
//
// A wave stages a tile of kNbSrTile entries in LDS with coalesced loads, then
// its 64/G lane groups each walk one run of U = kNbSrTile*G/64 consecutive
// entries.  Lane gl of a group owns V dense columns; per entry the group
// reads one contiguous piece of a row of X.  When the walk reaches the next
// row start the accumulator is flushed: plain store if the row lies inside
// the run, atomic add if it crosses the run's ends (prepare kernel, U).

constexpr int kNbSrTile = 512;
constexpr int kNbSrLogTile = 9;

template <int V>
__global__ __launch_bounds__(kBlock) void nb_sr_kernel(int M, int N, const int* __restrict__ rowptr,
                                                        const int* __restrict__ colidx,
                                                        const float* __restrict__ vals,
                                                        const float* __restrict__ X, float* __restrict__ Y,
                                                        int logG) {
    constexpr int T = kNbSrTile;
    __shared__ int s_col[kWavesPerBlock][T];
    __shared__ float s_val[kWavesPerBlock][T];
    __shared__ int s_win[kWavesPerBlock][T];
    const int lane = lane_id();
    const int wib = wave_in_block();
    int* cc = s_col[wib];
    float* cv = s_val[wib];
    int* win = s_win[wib];

    const int G = 1 << logG;
    const int gl = lane & (G - 1);
    const int g = lane >> logG;
    const int logU = kNbSrLogTile - 6 + logG;
    const unsigned U = 1u << logU;
    const long long n = ((long long)blockIdx.y * G + gl) * V;
    const bool col_ok = n < N;

    const TileRange tr = my_tiles<T>(rowptr, M);
    if (tr.first >= tr.last) return;
    const unsigned nnz = tr.nnz;

    int r_lo = wave_find_row(rowptr, M, tr.first * (unsigned)T, lane);
    unsigned rs_lo = (unsigned)rowptr[r_lo];

    for (unsigned tile = tr.first; tile < tr.last; ++tile) {
        const unsigned ts = tile * (unsigned)T;
        const unsigned te = (nnz - ts > (unsigned)T) ? ts + T : nnz;

        wave_lds_sync();                        // previous tile's readers are done
#pragma unroll
        for (int j = 0; j < T / kWave; ++j) {
            const int e = j * kWave + lane;
            const unsigned p = ts + (unsigned)e;
            if (p < te) { cc[e] = stream_load(colidx + p); cv[e] = stream_load(vals + p); }
        }
        const RowWindow w = build_row_window<T>(rowptr, M, win, r_lo, rs_lo, te, lane);   // syncs LDS

        const unsigned run_lo = ts + ((unsigned)g << logU);
        if (run_lo < te && col_ok) {
            const unsigned run_hi = (te - run_lo > U) ? run_lo + U : te;
            int cnt; unsigned rs, next;
            w.locate(run_lo, cnt, rs, next);     // row r_lo+cnt spans [rs, next)
            float acc[V];
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = 0.0f;

            for (unsigned p0 = run_lo; p0 < run_hi; p0 += 4) {
                float x[4][V]; float a[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned p = p0 + u;
                    if (p < run_hi) {
                        const int e = (int)(p - ts);
                        a[u] = cv[e];
                        load_vec<V>(X + (size_t)cc[e] * N + n, x[u]);
                    } else {
                        a[u] = 0.0f;
#pragma unroll
                        for (int i = 0; i < V; ++i) x[u][i] = 0.0f;
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const unsigned p = p0 + u;
                    if (p < run_hi) {
                        if (p == next) {
                            // row r_lo+cnt is complete as far as this run goes
                            float* y = Y + (size_t)((long long)r_lo + cnt) * N + n;
                            if (rs < run_lo) atomic_add_vec<V>(y, acc); else store_vec<V>(y, acc);
#pragma unroll
                            for (int i = 0; i < V; ++i) acc[i] = 0.0f;
                            do { ++cnt; rs = next; next = w.entry(cnt); } while (next <= p);   // skips empty rows
                        }
#pragma unroll
                        for (int i = 0; i < V; ++i) acc[i] = fmaf(a[u], x[u][i], acc[i]);
                    }
                }
            }
            float* y = Y + (size_t)((long long)r_lo + cnt) * N + n;
            if (rs < run_lo || next > run_hi) atomic_add_vec<V>(y, acc); else store_vec<V>(y, acc);
        }

        int lc; unsigned lrs, lre;
        w.locate(te - 1, lc, lrs, lre);
        r_lo = uniform(r_lo + lc);
        rs_lo = (unsigned)uniform((int)lrs);
    }
}

// ===========================================================================
// measurement aid: plain streaming copy
// ===========================================================================

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
