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
// loads / stores of V consecutive floats (V in {1, 2, 3, 4, 8}; V-float alignment assumed for 2, 4, 8)
// ---------------------------------------------------------------------------

template <int V>
__device__ __forceinline__ void load_vec(const float* __restrict__ p, float (&x)[V]) {
    if constexpr (V == 8) {                                  // two dwordx4 accesses
        const float4 t = *reinterpret_cast<const float4*>(p);
        const float4 u = *reinterpret_cast<const float4*>(p + 4);
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w; x[4] = u.x; x[5] = u.y; x[6] = u.z; x[7] = u.w;
    } else if constexpr (V == 4) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    } else if constexpr (V == 2) {
        const float2 t = *reinterpret_cast<const float2*>(p);
        x[0] = t.x; x[1] = t.y;
    } else if constexpr (V == 3) {
        __builtin_memcpy(&x[0], p, 12);
    } else {
        static_assert(V == 1, "unsupported width");
        x[0] = *p;
    }
}

template <int V>
__device__ __forceinline__ void store_vec(float* __restrict__ p, const float (&x)[V]) {
    if constexpr (V == 8) {
        *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
    } else if constexpr (V == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    } else if constexpr (V == 2) {
        *reinterpret_cast<float2*>(p) = make_float2(x[0], x[1]);
    } else if constexpr (V == 3) {
        __builtin_memcpy(p, &x[0], 12);
    } else {
        static_assert(V == 1, "unsupported width");
        *p = x[0];
    }
}

// The same for global addresses that are only known to be dword aligned (rows of a matrix whose leading
// dimension is not a multiple of V): still one dwordx2 / x3 / x4 access (two for V = 8), which the memory
// pipeline takes at any dword address; the compiler is merely told not to assume more.
// V = 8 is two groups of four; `second` says where the second group starts (4: right after the first; less:
// the two overlap, which is how the balanced parallel kernel takes N = 5, 6, 7 in one pass - the shared
// columns are then computed twice, identically, see second_half_own()).
template <int V>
__device__ __forceinline__ void load_vec_dword_aligned(const float* __restrict__ p, float (&x)[V], int second = 4) {
    if constexpr (V == 8) {
        __builtin_memcpy(&x[0], p, 16);
        __builtin_memcpy(&x[4], p + second, 16);
    } else {
        __builtin_memcpy(&x[0], p, sizeof(float) * V);
    }
}
template <int V>
__device__ __forceinline__ void store_vec_dword_aligned(float* __restrict__ p, const float (&x)[V], int second = 4) {
    if constexpr (V == 8) {
        __builtin_memcpy(p, &x[0], 16);
        __builtin_memcpy(p + second, &x[4], 16);      // overlapping columns hold equal values
    } else {
        __builtin_memcpy(p, &x[0], sizeof(float) * V);
    }
}

// Hardware fp32 add at the L2 (global_atomic_add_f32, no return value).
template <int V>
__device__ __forceinline__ void atomic_add_vec(float* p, const float (&x)[V]) {
#pragma unroll
    for (int i = 0; i < V; ++i) unsafeAtomicAdd(p + i, x[i]);
}
// V = 8 with the second group of four at `second` <= 4: every column exactly once
__device__ __forceinline__ void atomic_add_halves(float* p, const float (&x)[8], int second) {
#pragma unroll
    for (int i = 0; i < 4; ++i) unsafeAtomicAdd(p + i, x[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (second + i >= 4) unsafeAtomicAdd(p + second + i, x[4 + i]);
}

// The sparse arrays are read exactly once per call: mark the loads
// non-temporal so they do not push dense-matrix rows out of the caches.
__device__ __forceinline__ int stream_load(const int* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ float stream_load(const float* p) { return __builtin_nontemporal_load(p); }

// ---------------------------------------------------------------------------
// range-checked buffer accesses
// ---------------------------------------------------------------------------
//
// A buffer descriptor carries a base and a size; a lane whose byte offset falls
// outside reads zeros / writes nothing and causes no memory traffic.  That is
// predication without a branch: the instruction is always issued, so the
// outstanding-operation counter can be waited on exactly and later loads can
// stay in flight across it.  kOutOfRange switches a lane off.

constexpr unsigned kBufferFlags = 0x00020000u;      // raw 32-bit buffer descriptor, dword 3
constexpr unsigned kOutOfRange = 0xffffffffu;

// Bytes from the first element of a row-major matrix of `rows` rows, leading dimension `ld` and `cols`
// used columns to the end of its last row (a strided view stops there, not at rows * ld).
__host__ __device__ __forceinline__ unsigned long long dense_bytes(long long rows, long long ld, long long cols) {
    return rows > 0 ? (unsigned long long)((rows - 1) * ld + cols) * 4ull : 0ull;
}

// Descriptor for `bytes` bytes starting at p (clamped to the 4 GB a descriptor can span).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_buffer(const void* p, unsigned long long bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0,
                                             bytes > 0xffffffffull ? 0xffffffffu : (unsigned)bytes, kBufferFlags);
}

// Loads V consecutive floats at byte_offset; lanes whose offset is out of range get zeros and
// cause no memory traffic.  `aux` 2 marks the load non-temporal.
template <int V>
__device__ __forceinline__ void buffer_load_vec(__amdgpu_buffer_rsrc_t rsrc, unsigned byte_offset, float (&x)[V],
                                                int second_at = 4) {
    if constexpr (V == 8) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        // the second half of a switched-off lane stays out of range: 0xffffffff + 16 would wrap into it
        const unsigned second = byte_offset == kOutOfRange ? kOutOfRange : byte_offset + 4u * (unsigned)second_at;
        const f4 t = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_offset, 0, 0));
        const f4 u = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, second, 0, 0));
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w; x[4] = u.x; x[5] = u.y; x[6] = u.z; x[7] = u.w;
    } else if constexpr (V == 4) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const f4 t = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_offset, 0, 0));
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    } else if constexpr (V == 2) {
        typedef float f2 __attribute__((ext_vector_type(2)));
        const f2 t = __builtin_bit_cast(f2, __builtin_amdgcn_raw_buffer_load_b64(rsrc, byte_offset, 0, 0));
        x[0] = t.x; x[1] = t.y;
    } else if constexpr (V == 3) {
        typedef float f3 __attribute__((ext_vector_type(3)));
        // the whole vector changes type at once: taking the integer elements one by one and casting each made
        // the compiler load a single dword and copy it into all three
        const f3 t = __builtin_bit_cast(f3, __builtin_amdgcn_raw_buffer_load_b96(rsrc, byte_offset, 0, 0));
        x[0] = t.x; x[1] = t.y; x[2] = t.z;
    } else {
        static_assert(V == 1, "unsupported width");
        x[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, byte_offset, 0, 0));
    }
}

// AUX 2 marks the store non-temporal (the line need not stay in the L2).
template <int V, int AUX = 0>
__device__ __forceinline__ void buffer_store_vec(__amdgpu_buffer_rsrc_t rsrc, unsigned byte_offset, const float (&x)[V],
                                                 int second_at = 4) {
    if constexpr (V == 8) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        const unsigned second = byte_offset == kOutOfRange ? kOutOfRange : byte_offset + 4u * (unsigned)second_at;
        const f4 t = {x[0], x[1], x[2], x[3]};
        const f4 u = {x[4], x[5], x[6], x[7]};
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, t), rsrc, byte_offset, 0, AUX);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, u), rsrc, second, 0, AUX);
    } else if constexpr (V == 4) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        const f4 t = {x[0], x[1], x[2], x[3]};
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, t), rsrc, byte_offset, 0, AUX);
    } else if constexpr (V == 2) {
        typedef float f2 __attribute__((ext_vector_type(2)));
        typedef unsigned u2 __attribute__((ext_vector_type(2)));
        const f2 t = {x[0], x[1]};
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u2, t), rsrc, byte_offset, 0, AUX);
    } else if constexpr (V == 3) {
        typedef float f3 __attribute__((ext_vector_type(3)));
        typedef unsigned u3 __attribute__((ext_vector_type(3)));
        const f3 t = {x[0], x[1], x[2]};
        __builtin_amdgcn_raw_buffer_store_b96(__builtin_bit_cast(u3, t), rsrc, byte_offset, 0, AUX);
    } else {
        static_assert(V == 1, "unsupported width");
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, x[0]), rsrc, byte_offset, 0, AUX);
    }
}

// Scaling of a finished result (the kernels' AXPBY variants): v = alpha * v + beta * old.  With
// beta == 0 the old value is not read, so the output buffer may hold anything beforehand.
struct Scaling { float alpha, beta; };
template <int V, bool DWORD_ALIGNED = false>
__device__ __forceinline__ void scale_into(float (&v)[V], const float* __restrict__ old, Scaling s, int second_at = 4) {
    if (s.beta != 0.0f) {
        float o[V];
        if constexpr (DWORD_ALIGNED) load_vec_dword_aligned<V>(old, o, second_at); else load_vec<V>(old, o);
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] = fmaf(s.alpha, v[i], s.beta * o[i]);
    } else {
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] *= s.alpha;
    }
}
// the same with the old value behind a buffer descriptor (a switched-off lane reads zeros)
template <int V>
__device__ __forceinline__ void scale_into(float (&v)[V], __amdgpu_buffer_rsrc_t rsrc, unsigned byte_offset, Scaling s,
                                           int second_at = 4) {
    if (s.beta != 0.0f) {                           // wave-uniform
        float o[V];
        buffer_load_vec<V>(rsrc, byte_offset, o, second_at);
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] = fmaf(s.alpha, v[i], s.beta * o[i]);
    } else {
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] *= s.alpha;
    }
}

// Column index / value streams: non-temporal dword loads through a descriptor.
__device__ __forceinline__ int buffer_stream_i32(__amdgpu_buffer_rsrc_t r, unsigned byte_offset) {
    return (int)__builtin_amdgcn_raw_buffer_load_b32(r, byte_offset, 0, 2);
}
__device__ __forceinline__ float buffer_stream_f32(__amdgpu_buffer_rsrc_t r, unsigned byte_offset) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, byte_offset, 0, 2));
}

// ---------------------------------------------------------------------------
// the V dense columns of a lane in the sequential-reduction kernels
// ---------------------------------------------------------------------------
// Column block `block` covers `cols_per_block` columns (a multiple of V, at most G * V) from block * cols_per_block;
// lane `gl` of a group normally owns [first, first + V) with first = block * cols_per_block + gl * V.  RAGGED (N is
// not a multiple of V, N >= V): the lane whose window would pass N takes the last V columns of the row instead, so
// that every load stays inside the row; `skip` of them also belong to its left neighbour, which computes the same
// sums from the same entries in the same order - the lane keeps them out of what it adds to memory and of the
// scaled form's stores (plain stores may repeat them: the bits are the same).
struct LaneColumns {
    long long first;    // first column of the window
    int skip;           // leading columns of the window that are the neighbour's (0 < skip < V on one lane at most)
    bool any;           // the lane has columns at all
};
template <int V, bool RAGGED>
__device__ __forceinline__ LaneColumns lane_columns(unsigned block, int cols_per_block, int gl, int N) {
    LaneColumns c;
    c.first = (long long)block * cols_per_block + gl * V;
    c.skip = 0;
    c.any = gl * V < cols_per_block && c.first < N;
    if constexpr (RAGGED) {
        if (c.any && c.first + V > N) { c.skip = (int)(c.first + V - N); c.first = (long long)N - V; }
    }
    return c;
}

// Stores a lane's V results at byte_offset (kOutOfRange: nothing).  With RAGGED the last lane of a row shares its
// first `skip` columns with its neighbour, and both hold the same bits there (the same entries in the same order
// went into them).  In the plain product both may store them: whichever write lands last changes nothing, also
// when the neighbour sits in another column block and writes at another time.  LEAVE_SHARED_OUT (the scaled form,
// where a result depends on the old Y and the neighbour may have replaced that already): the lane with skip != 0
// stores exactly its last `tail` = N % V values (wave-uniform) in one more store of that width, issued by the
// whole wave and switched off everywhere else.
template <int V, bool RAGGED, int AUX = 0, bool LEAVE_SHARED_OUT = true>
__device__ __forceinline__ void buffer_store_columns(__amdgpu_buffer_rsrc_t rsrc, unsigned byte_offset, const float (&x)[V],
                                                     int skip, int tail) {
    if constexpr (!RAGGED || !LEAVE_SHARED_OUT) {
        buffer_store_vec<V, AUX>(rsrc, byte_offset, x);
    } else {
        static_assert(V == 4, "the shared lane exists at four columns per lane only");
        buffer_store_vec<V, AUX>(rsrc, skip == 0 ? byte_offset : kOutOfRange, x);
        const bool on = skip != 0 && byte_offset != kOutOfRange;
        if (tail == 1) {
            const float t[1] = {x[3]};
            buffer_store_vec<1, AUX>(rsrc, on ? byte_offset + 12u : kOutOfRange, t);
        } else if (tail == 2) {
            const float t[2] = {x[2], x[3]};
            buffer_store_vec<2, AUX>(rsrc, on ? byte_offset + 8u : kOutOfRange, t);
        } else {
            const float t[3] = {x[1], x[2], x[3]};
            buffer_store_vec<3, AUX>(rsrc, on ? byte_offset + 4u : kOutOfRange, t);
        }
    }
}

// ---------------------------------------------------------------------------
// wave64 segmented inclusive scan on DPP (vectorized segment reduction,
// paper Section 2.1.1)
// ---------------------------------------------------------------------------
//
// The paper runs a prefix-sum network over the lanes of a warp in which two
// elements are added only if they carry the same row index.  Along a run of
// CSR entries row indices never decrease, so two lanes share a row exactly
// when no segment head lies between them.  Each lane therefore needs one number,
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
constexpr int kDppWaveShr1 = 0x138;   // lane l reads lane l-1 across the whole wave; lane 0 gets the fill value

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

// Inclusive running maximum over the lanes of a wave (same DPP network, no
// segments): lane l gets max(v[0..l]).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned dpp_or_zero_u(unsigned v) {
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}

__device__ __forceinline__ unsigned wave_max_scan(unsigned v) {
    unsigned t;
    t = dpp_or_zero_u<kDppRowShr1, 0xf>(v); v = t > v ? t : v;
    t = dpp_or_zero_u<kDppRowShr2, 0xf>(v); v = t > v ? t : v;
    t = dpp_or_zero_u<kDppRowShr4, 0xf>(v); v = t > v ? t : v;
    t = dpp_or_zero_u<kDppRowShr8, 0xf>(v); v = t > v ? t : v;
    t = dpp_or_zero_u<kDppRowBcast15, 0xa>(v); v = t > v ? t : v;
    t = dpp_or_zero_u<kDppRowBcast31, 0xc>(v); v = t > v ? t : v;
    return v;
}

}  // namespace dgsp
