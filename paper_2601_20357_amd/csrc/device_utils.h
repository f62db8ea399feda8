// Device-side helpers shared by the TABED kernels: wave64 / workgroup reductions,
// Philox4x32-10, guarded vector loads.  gfx950 only (wavefront = 64 lanes).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "internal.h"

namespace tabed {

constexpr float kMargin = 1e-6f;        // decisions closer than this (relative) are flagged

// ---------------------------------------------------------------- wave64 reductions (deterministic order)
// Four DPP steps (lane^1, lane^2, mirror within 8, mirror within 16) leave every lane of a 16-lane row with
// the row's result; the four row results are then read as scalars (v_readlane) and combined in row order.
// No LDS traffic and no index registers, unlike ds_bpermute-based shuffles.
constexpr int kDppXor1 = 0xB1;          // quad_perm:[1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i <- lane 7 - i   (within 8)
constexpr int kDppMirror = 0x140;       // lane i <- lane 15 - i  (within 16)

template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __builtin_bit_cast(float, dpp_i32<CTRL>(__builtin_bit_cast(int, v)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const long long b = __builtin_bit_cast(long long, v);
    const unsigned lo = (unsigned)dpp_i32<CTRL>((int)(unsigned)b), hi = (unsigned)dpp_i32<CTRL>((int)(unsigned)(b >> 32));
    return __builtin_bit_cast(double, (long long)(((unsigned long long)hi << 32) | lo));
}
__device__ __forceinline__ float lane_f32(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ double lane_f64(double v, int lane) {
    const long long b = __builtin_bit_cast(long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), lane);
    return __builtin_bit_cast(double, (long long)(((unsigned long long)hi << 32) | lo));
}

__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<kDppXor1>(v));
    v = fmaxf(v, dpp_f32<kDppXor2>(v));
    v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_f32<kDppMirror>(v));
    return fmaxf(fmaxf(lane_f32(v, 0), lane_f32(v, 16)), fmaxf(lane_f32(v, 32), lane_f32(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f32<kDppXor1>(v);
    v += dpp_f32<kDppXor2>(v);
    v += dpp_f32<kDppHalfMirror>(v);
    v += dpp_f32<kDppMirror>(v);
    return (lane_f32(v, 0) + lane_f32(v, 16)) + (lane_f32(v, 32) + lane_f32(v, 48));
}
__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_f64<kDppXor1>(v);
    v += dpp_f64<kDppXor2>(v);
    v += dpp_f64<kDppHalfMirror>(v);
    v += dpp_f64<kDppMirror>(v);
    return (lane_f64(v, 0) + lane_f64(v, 16)) + (lane_f64(v, 32) + lane_f64(v, 48));
}

// Workgroup reductions over kBlock threads through a 4-entry LDS array.  Two barriers each, so the
// scratch array can be reused by the next call.
__device__ __forceinline__ float block_max(float v, float* lds4) {
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = fmaxf(fmaxf(lds4[0], lds4[1]), fmaxf(lds4[2], lds4[3]));
    __syncthreads();
    return r;
}
__device__ __forceinline__ double block_sum(double v, double* lds4) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
    __syncthreads();
    return r;
}

// Inclusive prefix sum across the 64 lanes of a wave, fixed order, no LDS traffic: Hillis-Steele inside each
// 16-lane row with row_shr (lanes shifted in from outside the row read 0), then the total of row 0 goes to
// row 1 and that of row 2 to row 3 (row_bcast:15), then the total of rows 0-1 goes to rows 2-3 (row_bcast:31).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64_zero(double v) {
    const long long b = __builtin_bit_cast(long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)b, CTRL, ROW_MASK, 0xF, true);
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(b >> 32), CTRL, ROW_MASK, 0xF, true);
    return __builtin_bit_cast(double, (long long)(((unsigned long long)hi << 32) | lo));
}
__device__ __forceinline__ double wave_inclusive_scan(double v) {
    v += dpp_f64_zero<0x111, 0xF>(v);    // row_shr:1
    v += dpp_f64_zero<0x112, 0xF>(v);    // row_shr:2
    v += dpp_f64_zero<0x114, 0xF>(v);    // row_shr:4
    v += dpp_f64_zero<0x118, 0xF>(v);    // row_shr:8
    v += dpp_f64_zero<0x142, 0xA>(v);    // row_bcast:15 into rows 1 and 3
    v += dpp_f64_zero<0x143, 0xC>(v);    // row_bcast:31 into rows 2 and 3
    return v;
}

// Exclusive prefix of one value per thread over the whole workgroup, in thread order; *total = sum.
__device__ __forceinline__ double block_exclusive_scan(double v, double* lds4, double* total) {
    double inc = wave_inclusive_scan(v);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 63) lds4[w] = inc;
    __syncthreads();
    double base = 0.0;
    for (int i = 0; i < w; ++i) base += lds4[i];
    *total = ((lds4[0] + lds4[1]) + lds4[2]) + lds4[3];
    __syncthreads();
    return base + inc - v;
}

__device__ __forceinline__ int wave_min_i32(int v) {
    v = min(v, dpp_i32<kDppXor1>(v));
    v = min(v, dpp_i32<kDppXor2>(v));
    v = min(v, dpp_i32<kDppHalfMirror>(v));
    v = min(v, dpp_i32<kDppMirror>(v));
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
__device__ __forceinline__ int wave_max_i32(int v) {
    v = max(v, dpp_i32<kDppXor1>(v));
    v = max(v, dpp_i32<kDppXor2>(v));
    v = max(v, dpp_i32<kDppHalfMirror>(v));
    v = max(v, dpp_i32<kDppMirror>(v));
    return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
// Smallest `first_key` over the workgroup (keys order the candidates along the prefix); if no thread offers
// one (first_key = INT_MAX everywhere), the largest `last_key`; -1 if there is none either.
__device__ __forceinline__ int block_pick_key(int first_key, int last_key, int* lds_first4, int* lds_last4) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int f = wave_min_i32(first_key), l = wave_max_i32(last_key);
    if (lane == 0) { lds_first4[w] = f; lds_last4[w] = l; }
    __syncthreads();
    const int first = min(min(lds_first4[0], lds_first4[1]), min(lds_first4[2], lds_first4[3]));
    const int last = max(max(lds_last4[0], lds_last4[1]), max(lds_last4[2], lds_last4[3]));
    __syncthreads();
    return first != 0x7fffffff ? first : last;
}

// Which thread's run of the prefix contains `target`?  Every thread passes the exclusive prefix and the
// sum of its run (block_exclusive_scan order).  Returns the lowest thread whose inclusive prefix exceeds
// target; if rounding lets none exceed it, the highest thread with a non-empty run; -1 if all runs are
// empty.  Ballots and two small LDS arrays: no same-address atomics.
__device__ __forceinline__ int block_find_owner(double excl, double run, double target, int* lds_first4,
                                                int* lds_last4) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const unsigned long long cross = __ballot(run > 0.0 && excl + run > target);
    const unsigned long long live = __ballot(run > 0.0);
    if (lane == 0) {
        lds_first4[w] = cross ? (w * 64 + __ffsll((long long)cross) - 1) : 0x7fffffff;
        lds_last4[w] = live ? (w * 64 + 63 - __clzll((long long)live)) : -1;
    }
    __syncthreads();
    const int first = min(min(lds_first4[0], lds_first4[1]), min(lds_first4[2], lds_first4[3]));
    const int last = max(max(lds_last4[0], lds_last4[1]), max(lds_last4[2], lds_last4[3]));
    __syncthreads();
    return first != 0x7fffffff ? first : last;
}

// ---------------------------------------------------------------- publishing partial results across workgroups
// "Last workgroup done" hand-over without an agent-scope fence.  On gfx950 such a fence writes back and
// invalidates the whole L2 of the XCD (measured 2-3 us per fence inside these kernels).  What a release /
// acquire pair has to guarantee here is narrower: (1) the partial results are at the device's coherence point
// before the arrival counter moves, and (2) the finishing workgroup does not read them from a stale cache
// line.  Both follow from the instructions themselves:
//   * publish_store() is an agent-scope atomic store: it is emitted as a write-through store (sc1) that
//     is acknowledged only once it has reached the memory side shared by all XCDs; nothing published is
//     ever left dirty in an XCD's L2, which is all the fence's write-back would be for.
//   * publish_barrier(): every thread waits until ALL of its outstanding vector-memory operations have been
//     acknowledged (s_waitcnt vmcnt(0): on gfx9 the counter covers stores as well as loads), then the
//     workgroup meets.  A plain __syncthreads() does not wait for stores.
//   * arrive() is an agent-scope atomic add issued after that barrier, so it is ordered after every
//     published store of the workgroup; the workgroup whose add returns the final count reads the partial
//     results with published_load() only, an agent-scope atomic load (sc1) that is served from the
//     coherence point, never from a line an XCD cached earlier; those loads are issued after the add has
//     returned (its value decides the branch).
// What would break it: a publish_store() that is not waited for before the barrier, an ordinary load of
// published data in the finishing workgroup, or an ordinary store of data another workgroup then reads.
__device__ __forceinline__ void publish_barrier() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}
__device__ __forceinline__ void publish_store(double* p, double v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_store(int* p, int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double published_load(const double* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float published_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int published_load(const int* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Returns true in the workgroup whose arrival completes `expected`; that workgroup also re-arms the counter.
__device__ __forceinline__ bool arrive(uint32_t* counter, uint32_t expected) {
    const uint32_t old = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old != expected - 1) return false;
    __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// ---------------------------------------------------------------- arg-max with runner-up
struct Top2 {
    float v1;  // maximum
    int i1;    // its lowest index
    float v2;  // largest value among all other elements
};
__device__ __forceinline__ Top2 top2_empty() { return Top2{-INFINITY, 0x7fffffff, -INFINITY}; }
__device__ __forceinline__ Top2 top2_merge(const Top2& a, const Top2& b) {
    const bool b_wins = (b.v1 > a.v1) || (b.v1 == a.v1 && b.i1 < a.i1);
    Top2 r;
    if (b_wins) { r.v1 = b.v1; r.i1 = b.i1; r.v2 = fmaxf(a.v1, b.v2); }
    else        { r.v1 = a.v1; r.i1 = a.i1; r.v2 = fmaxf(a.v2, b.v1); }
    return r;
}
__device__ __forceinline__ Top2 top2_push(const Top2& a, float x, int idx) {
    return top2_merge(a, Top2{x, idx, -INFINITY});
}
template <int CTRL>
__device__ __forceinline__ Top2 top2_dpp_step(const Top2& t) {
    return top2_merge(t, Top2{dpp_f32<CTRL>(t.v1), dpp_i32<CTRL>(t.i1), dpp_f32<CTRL>(t.v2)});
}
__device__ __forceinline__ Top2 top2_at(const Top2& t, int lane) {
    return Top2{lane_f32(t.v1, lane), __builtin_amdgcn_readlane(t.i1, lane), lane_f32(t.v2, lane)};
}
// NB: merging a candidate with a copy of itself must not happen (it would count the maximum as its own
// runner-up); the DPP steps below always pair disjoint lane groups.
__device__ __forceinline__ Top2 wave_top2(Top2 t) {
    t = top2_dpp_step<kDppXor1>(t);
    t = top2_dpp_step<kDppXor2>(t);
    t = top2_dpp_step<kDppHalfMirror>(t);
    t = top2_dpp_step<kDppMirror>(t);
    return top2_merge(top2_merge(top2_at(t, 0), top2_at(t, 16)), top2_merge(top2_at(t, 32), top2_at(t, 48)));
}

// Plain (value, lowest index) arg-max.
struct ArgMax {
    float v;
    int i;
};
__device__ __forceinline__ ArgMax argmax_merge(const ArgMax& a, const ArgMax& b) {
    return ((b.v > a.v) || (b.v == a.v && b.i < a.i)) ? b : a;
}
template <int CTRL>
__device__ __forceinline__ ArgMax argmax_dpp_step(const ArgMax& t) {
    return argmax_merge(t, ArgMax{dpp_f32<CTRL>(t.v), dpp_i32<CTRL>(t.i)});
}
__device__ __forceinline__ ArgMax argmax_at(const ArgMax& t, int lane) {
    return ArgMax{lane_f32(t.v, lane), __builtin_amdgcn_readlane(t.i, lane)};
}
__device__ __forceinline__ ArgMax wave_argmax(ArgMax t) {
    t = argmax_dpp_step<kDppXor1>(t);
    t = argmax_dpp_step<kDppXor2>(t);
    t = argmax_dpp_step<kDppHalfMirror>(t);
    t = argmax_dpp_step<kDppMirror>(t);
    return argmax_merge(argmax_merge(argmax_at(t, 0), argmax_at(t, 16)), argmax_merge(argmax_at(t, 32), argmax_at(t, 48)));
}

// ---------------------------------------------------------------- Philox4x32-10 (Salmon et al., SC'11)
struct U4 {
    uint32_t x, y, z, w;
};
__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                             uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}
__device__ __forceinline__ float u01(uint32_t x) { return (float)(x >> 8) * (1.0f / 16777216.0f); }

// Uniform of (seed, round, b, pos): word 0 or 1 of the Philox block.
__device__ __forceinline__ float tabed_uniform(uint64_t seed, uint64_t round, uint32_t b, uint32_t pos, int word) {
    U4 r = philox4x32_10((uint32_t)round, (uint32_t)(round >> 32), b, pos, (uint32_t)seed, (uint32_t)(seed >> 32));
    return u01(word == 0 ? r.x : r.y);
}

// ---------------------------------------------------------------- guarded row loads
// Four consecutive logits starting at element v (v % 4 == 0) of a row of V floats; elements past the end
// of the row come back as -inf.  VEC needs V % 4 == 0 and a 16-byte aligned row.
template <bool VEC>
__device__ __forceinline__ float4 load4(const float* __restrict__ row, int v, int V) {
    const float ninf = -INFINITY;
    if (VEC) {
        if (v < V) return *reinterpret_cast<const float4*>(row + v);
        return make_float4(ninf, ninf, ninf, ninf);
    }
    float4 r;
    r.x = (v + 0 < V) ? row[v + 0] : ninf;
    r.y = (v + 1 < V) ? row[v + 1] : ninf;
    r.z = (v + 2 < V) ? row[v + 2] : ninf;
    r.w = (v + 3 < V) ? row[v + 3] : ninf;
    return r;
}

__device__ __forceinline__ float f4get(const float4& a, int e) { return e == 0 ? a.x : e == 1 ? a.y : e == 2 ? a.z : a.w; }

}  // namespace tabed
