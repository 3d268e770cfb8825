// Device-side building blocks shared by the four CSR kernels (gfx950, wave64).
//
// Nothing here is generic GPU code: lane counts, DPP controls and the
// XCD-aware block mapping are those of CDNA4.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dgsp {

constexpr int kWave = 64;                       // lanes per wavefront
constexpr int kBlock = 256;                     // threads per workgroup
constexpr int kWavesPerBlock = kBlock / kWave;  // 4, one per SIMD
constexpr unsigned kXcd = 8;                    // accelerator dies, each with its own L2

// ---------------------------------------------------------------------------
// wave-level plumbing
// ---------------------------------------------------------------------------

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// threadIdx.x / 64, forced into an SGPR so that everything derived from it is
// known to be wave-uniform.
__device__ __forceinline__ int wave_in_block() {
    return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
}

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ int read_lane(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ float read_lane(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// Orders LDS traffic between the lanes of ONE wave.  A wave's LDS
// instructions are executed in program order, so no hardware barrier is
// needed; this only stops the compiler from moving LDS reads above the writes
// (or the next round's writes above this round's reads).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroups are dealt round-robin to the 8 XCDs (block b runs on XCD b % 8).
// This maps b to a logical id such that every XCD owns one contiguous range of
// logical ids: neighbouring rows / tiles then share one L2 instead of eight.
// Bijective on [0, nb) for any nb.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned b, unsigned nb) {
    const unsigned q = nb / kXcd, r = nb % kXcd;
    const unsigned x = b % kXcd, i = b / kXcd;
    return x * q + (x < r ? x : r) + i;
}

// ---------------------------------------------------------------------------
// loads / stores of V consecutive floats (V in {1, 2, 4})
// ---------------------------------------------------------------------------

template <int V>
__device__ __forceinline__ void load_vec(const float* __restrict__ p, float (&x)[V]) {
    if constexpr (V == 4) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    } else if constexpr (V == 2) {
        const float2 t = *reinterpret_cast<const float2*>(p);
        x[0] = t.x; x[1] = t.y;
    } else {
        x[0] = *p;
    }
}

template <int V>
__device__ __forceinline__ void store_vec(float* __restrict__ p, const float (&x)[V]) {
    if constexpr (V == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    } else if constexpr (V == 2) {
        *reinterpret_cast<float2*>(p) = make_float2(x[0], x[1]);
    } else {
        *p = x[0];
    }
}

// Hardware fp32 add at the L2 (global_atomic_add_f32, no return value).
template <int V>
__device__ __forceinline__ void atomic_add_vec(float* p, const float (&x)[V]) {
#pragma unroll
    for (int i = 0; i < V; ++i) unsafeAtomicAdd(p + i, x[i]);
}

// The sparse arrays are read exactly once per call: mark the loads
// non-temporal so they do not push dense-matrix rows out of the caches.
__device__ __forceinline__ int stream_load(const int* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ float stream_load(const float* p) { return __builtin_nontemporal_load(p); }

// ---------------------------------------------------------------------------
// wave64 segmented inclusive scan on DPP (vectorized segment reduction,
// paper Section 2.1.1)
// ---------------------------------------------------------------------------
//
// The paper runs a prefix-sum network over the lanes of a warp whose
// operator is "add if the two elements carry the same row index".  Along a
// run of CSR entries row indices never decrease, so "same row" is the same as
// "no segment head in between".  Each lane therefore needs one number,
//     h = how many lanes directly below it belong to its segment,
// and a partner at distance d is added iff h >= d.  The network is the
// canonical gfx9 wave64 scan: row_shr 1,2,4,8 inside each row of 16 lanes,
// then row_bcast:15 (lane 15 of a row to the next row) and row_bcast:31
// (lane 31 to the upper half).  Six data-parallel-primitive moves, no LDS.
// After the scan lane l holds the sum over lanes [l-h, l]; the last lane of a
// segment holds the segment total.

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or_zero(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false));
}

constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;

// `width` (wave-uniform, a power of two <= 64) promises h < width, which lets
// the steps with d >= width be skipped by a scalar branch.
template <int V>
__device__ __forceinline__ void segmented_scan(float (&v)[V], int h, int lane, int width = kWave) {
    const bool c1 = h >= 1, c2 = h >= 2, c4 = h >= 4, c8 = h >= 8;
    const bool c16 = h >= (lane & 15) + 1;   // my segment reaches into the previous row of 16
    const bool c32 = h >= lane - 31;         // ... into the lower half (false for lanes < 32 only if h < 0)
    if (width > 1) {
#pragma unroll
        for (int i = 0; i < V; ++i) { const float t = dpp_or_zero<kDppRowShr1, 0xf>(v[i]); v[i] += c1 ? t : 0.0f; }
    }
    if (width > 2) {
#pragma unroll
        for (int i = 0; i < V; ++i) { const float t = dpp_or_zero<kDppRowShr2, 0xf>(v[i]); v[i] += c2 ? t : 0.0f; }
    }
    if (width > 4) {
#pragma unroll
        for (int i = 0; i < V; ++i) { const float t = dpp_or_zero<kDppRowShr4, 0xf>(v[i]); v[i] += c4 ? t : 0.0f; }
    }
    if (width > 8) {
#pragma unroll
        for (int i = 0; i < V; ++i) { const float t = dpp_or_zero<kDppRowShr8, 0xf>(v[i]); v[i] += c8 ? t : 0.0f; }
    }
    if (width > 16) {
#pragma unroll
        for (int i = 0; i < V; ++i) { const float t = dpp_or_zero<kDppRowBcast15, 0xa>(v[i]); v[i] += c16 ? t : 0.0f; }
    }
    if (width > 32) {
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float t = dpp_or_zero<kDppRowBcast31, 0xc>(v[i]);
            v[i] += (lane >= 32 && c32) ? t : 0.0f;
        }
    }
}

// ---------------------------------------------------------------------------
// locating CSR rows from positions (nnz-balanced kernels)
// ---------------------------------------------------------------------------
//
// The paper's balanced kernels refer "to the row indices of each element"
// (Section 2.1.1) without saying where they come from.  The ABI passes only
// rowptr, so rows are found by searching it.

// Largest row r in [0, M) with rowptr[r] <= pos.  Needs rowptr[0] <= pos <
// rowptr[M].  All 64 lanes probe at once, so each round divides the range by
// 64: four rounds for a million rows.  Result is wave-uniform.
__device__ __forceinline__ int wave_find_row(const int* __restrict__ rowptr, int M, unsigned pos, int lane) {
    int lo = 0, hi = M;   // invariant: rowptr[lo] <= pos < rowptr[hi]
    while (hi - lo > 1) {
        const int span = hi - lo;
        const int step = (span + 63) >> 6;
        int idx = lo + lane * step;
        idx = idx < hi ? idx : hi;
        const unsigned v = (unsigned)rowptr[idx];
        const unsigned long long below = __ballot(v <= pos);   // 1...10...0, lane 0 always set
        int cnt = __popcll(below);
        cnt = cnt > 0 ? cnt : 1;                               // only a malformed rowptr gives 0
        const int nlo = lo + (cnt - 1) * step;
        int nhi = lo + cnt * step;
        nhi = nhi < hi ? nhi : hi;
        lo = nlo;
        hi = nhi;
    }
    return uniform(lo);
}

// A wave's view of the row starts that follow row `r_lo`:
//   entry i  ==  rowptr[min(r_lo + 1 + i, M)]
// kept in LDS (`win`, WMAX ints) when the first `wlen` entries already reach
// past the end of the tile (`covered`), else read from global memory.
struct RowWindow {
    const int* __restrict__ rowptr;
    const int* win;    // LDS
    int M;
    int r_lo;          // wave-uniform; rowptr[r_lo] <= first position of the tile
    unsigned rs_lo;    // rowptr[r_lo]
    int wlen;          // entries valid in win (multiple of 64)
    bool covered;      // win[wlen-1] >= tile end

    __device__ __forceinline__ unsigned entry(int i) const {
        if (covered) return (unsigned)win[i];
        long long r = (long long)r_lo + 1 + i;
        return (unsigned)rowptr[r < M ? r : M];
    }

    // For a position p inside the tile: cnt = number of entries <= p, so that
    // p lies in row r_lo + cnt, which spans [rs, re).
    __device__ __forceinline__ void locate(unsigned p, int& cnt, unsigned& rs, unsigned& re) const {
        int c = 0;
        if (covered) {
            // branch-free upper bound over win[0, wlen); win[wlen-1] > p
            for (int s = 256; s >= 64; s >>= 1) {           // only when the window grew past 64
                if (s < wlen) { if (c + s - 1 < wlen && (unsigned)win[c + s - 1] <= p) c += s; }
            }
#pragma unroll
            for (int s = 32; s >= 1; s >>= 1) {
                if ((unsigned)win[c + s - 1] <= p) c += s;
            }
            rs = c ? (unsigned)win[c - 1] : rs_lo;
            re = (unsigned)win[c];
        } else {
            // first index in (r_lo, M] whose row start exceeds p; rowptr[M] = nnz > p
            int lo = r_lo + 1, hi = M;
            while (lo < hi) {
                const int mid = lo + ((hi - lo) >> 1);
                if ((unsigned)rowptr[mid] <= p) lo = mid + 1; else hi = mid;
            }
            c = lo - 1 - r_lo;
            rs = (unsigned)rowptr[lo - 1];
            re = (unsigned)rowptr[lo];
        }
        cnt = c;
    }
};

// Fills the LDS window for the tile [ts, te) (all lanes of the wave call
// this).  WMAX is a multiple of 64, at most 512.
template <int WMAX>
__device__ __forceinline__ RowWindow build_row_window(const int* __restrict__ rowptr, int M, int* win,
                                                      int r_lo, unsigned rs_lo, unsigned te, int lane) {
    RowWindow w;
    w.rowptr = rowptr; w.win = win; w.M = M; w.r_lo = r_lo; w.rs_lo = rs_lo;
    int wlen = 0;
    bool covered;
    wave_lds_sync();   // the previous tile's readers are done with `win`
    do {
        long long r = (long long)r_lo + 1 + wlen + lane;
        const int v = rowptr[r < M ? r : M];
        win[wlen + lane] = v;
        wlen += kWave;
        covered = (unsigned)read_lane(v, kWave - 1) >= te;
    } while (!covered && wlen < WMAX);
    wave_lds_sync();
    w.wlen = wlen; w.covered = covered;
    return w;
}

}  // namespace dgsp
