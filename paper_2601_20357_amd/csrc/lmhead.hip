// LM head of the n batched drafts (Alg. 1 line 5, last layer of the shared draft model):
//   L[r, v] = sum_k H[r, k] * W[v, k],   r = b*n + j  (M = n*B rows),
// with the first half of the per-draft softmax fused into the epilogue: for every row and every 32-wide
// vocabulary tile the kernel also writes  pm = max_v s(v)  and  ps = sum_v exp(s(v) - pm),  s = L / T_b.
// gfx950: bf16 operands go through v_mfma_f32_32x32x16_bf16 (fp32 accumulate); fp32 operands (the tiny
// correctness configuration) use plain FMAs.
#include <hip/hip_bf16.h>

#include <mutex>
#include <type_traits>

#include "device_utils.h"
#include "internal.h"

namespace tabed {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float row_inv_temperature(const float* temperature, int row, int n) {
    const float T = temperature[row / n];
    return (T > 0.f) ? 1.f / T : 1.f;
}

// Reductions over the 32 lanes that share lane/32 (xor offsets < 32 never leave the half-wave).
__device__ __forceinline__ float half_max(float v) {
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float half_sum(float v) {
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Epilogue of one 32x32 accumulator tile: lane holds column (lane % 32) and the 16 rows
// 8*(r/4) + 4*(lane/32) + r%4 of the block that starts at row m_base.  Writes logits and the tile's softmax
// partials.  inv_t[i] = 1/T of row m_table0 + i (an LDS table filled by the caller).
__device__ __forceinline__ void store_tile_32x32(const f32x16& acc, int m_base, int v_base, int M, int V, int NT,
                                                 const float* inv_t, int m_table0, float* __restrict__ L,
                                                 float* __restrict__ pm, float* __restrict__ ps) {
    if (v_base >= V) return;
    const int lane = threadIdx.x & 63;
    const int col = lane & 31, half = lane >> 5;
    const int v = v_base + col;
    const int tile = v_base / kTileV;
    const bool vlive = (v < V);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = m_base + 8 * (r / 4) + 4 * half + (r % 4);
        const bool live = (m < M);          // uniform over the half-wave
        const float x = acc[r];
        float s = -INFINITY;
        if (live && vlive) {
            L[(size_t)m * V + v] = x;
            s = x * inv_t[m - m_table0];
        }
        const float mx = half_max(s);
        const float e = (s > -INFINITY) ? __expf(s - mx) : 0.f;
        const float sum = half_sum(e);
        if (live && col == 0) {
            pm[(size_t)m * NT + tile] = mx;
            ps[(size_t)m * NT + tile] = sum;
        }
    }
}

// Epilogue of one 32x32 accumulator tile held TRANSPOSED: lane holds result row m_base + lane % 32 and the 16
// vocabulary entries v_base + 8*(r/4) + 4*(lane/32) + r%4.  The softmax partials of a row are then a
// 16-value in-register reduction plus one exchange between the two half-waves, and every lane stores four
// runs of four consecutive logits.  inv_t[m] = 1/T of row m (LDS table).  With `pstage` the partials go to an
// LDS table instead, from which the caller writes a workgroup's four tiles of a row as one 16-byte store.
// PUB: the logits are read again inside this kernel, by the workgroup that finishes the launch (fused sampler): they
// are then stored write-through at device scope (still streaming past L2) instead of as plain streaming stores.
template <bool PUB = false>
__device__ __forceinline__ void store_tile_32x32_t(const f32x16& acc, int m_base, int v_base, int M, int V, int NT,
                                                   const float* inv_t, float* __restrict__ L,
                                                   float* __restrict__ pm, float* __restrict__ ps,
                                                   unsigned char* tpatch, float* pstage = nullptr, int pslot = 0) {
    if (v_base >= V) return;
    const int lane = threadIdx.x & 63;
    const int col = lane & 31, half = lane >> 5;
    const int m = m_base + col;
    const bool live = (m < M);
    const float it = live ? inv_t[m] : 1.f;
    float sc[16];
    float mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int v = v_base + 8 * (r / 4) + 4 * half + (r % 4);
        sc[r] = (live && v < V) ? acc[r] * it : -INFINITY;
        mx = fmaxf(mx, sc[r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += (sc[r] > -INFINITY) ? __expf(sc[r] - mx) : 0.f;
    sum += __shfl_xor(sum, 32);
    if (live && half == 0) {
        if (pstage != nullptr) {                    // collected per workgroup: [array][row][tile of the group]
            pstage[(0 * 64 + m) * 4 + pslot] = mx;
            pstage[(1 * 64 + m) * 4 + pslot] = sum;
        } else {
            pm[(size_t)m * NT + v_base / kTileV] = mx;
            ps[(size_t)m * NT + v_base / kTileV] = sum;
        }
    }
    if ((V & 3) == 0 && v_base + 32 <= V) {
        // Full tile: turn the block through the wave's LDS patch ([32 rows][32 v] floats, 144-byte rows) so
        // that 8 lanes store one whole 128-byte line of a row, and stream it past L2: the logits are next
        // read tens of megabytes later, and full-line streaming stores measured 1.9 us faster per launch
        // than leaving 8 MB of dirty partial lines to the end-of-kernel write-back.
#pragma unroll
        for (int g = 0; g < 4; ++g)
            *reinterpret_cast<float4*>(tpatch + col * 144 + (8 * g + 4 * half) * 4) =
                make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int mr = 8 * i + (lane >> 3), q = lane & 7;
            const float4 val = *reinterpret_cast<const float4*>(tpatch + mr * 144 + q * 16);
            if (m_base + mr < M) {
                if (PUB) {
                    // buffer store with the "nt sc1" cache policy (aux bits 1 and 4): streaming and written through
                    // to device scope; the compiler counts it like any other vector-memory store
                    const __amdgpu_buffer_rsrc_t rs =
                        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(L), 0, M * V * 4, 0x00020000);
                    __builtin_amdgcn_raw_buffer_store_b128(
                        u32x4{__builtin_bit_cast(uint32_t, val.x), __builtin_bit_cast(uint32_t, val.y),
                              __builtin_bit_cast(uint32_t, val.z), __builtin_bit_cast(uint32_t, val.w)},
                        rs, ((m_base + mr) * V + v_base + 4 * q) * 4, 0, 18);
                } else {
                    __builtin_nontemporal_store(f32x4{val.x, val.y, val.z, val.w},
                                                reinterpret_cast<f32x4*>(L + (size_t)(m_base + mr) * V + v_base + 4 * q));
                }
            }
        }
        return;
    }
    if (!live) return;
    float* row = L + (size_t)m * V;                // ragged last tile or unaligned rows: element-wise
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int v = v_base + 8 * g + 4 * half + e;
            if (v < V) {
                if (PUB) publish_store(&row[v], acc[4 * g + e]);
                else row[v] = acc[4 * g + e];
            }
        }
}

// ---------------------------------------------------------------- bf16, any shape: LDS-tiled MFMA GEMM
// Workgroup tile 64 (rows) x 64 (vocabulary) x 64 (k); wave w owns the 32x32 quadrant (w/2, w%2).
// Both operands are K-contiguous in memory, which is exactly the per-lane 8-element run the MFMA wants,
// so LDS only transposes "who holds which row".  Rows are padded by 16 bytes against bank conflicts.
constexpr int kBM = 64, kBN = 64, kBK = 64, kPad = 8;

__global__ __launch_bounds__(kBlock) void k_lmhead_bf16(int M, int d, int V, int n, int NT,
                                                        const __hip_bfloat16* __restrict__ W,
                                                        const __hip_bfloat16* __restrict__ H,
                                                        const float* __restrict__ temperature,
                                                        float* __restrict__ L, float* __restrict__ pm,
                                                        float* __restrict__ ps) {
    __shared__ __attribute__((aligned(16))) uint16_t sA[kBM][kBK + kPad];
    __shared__ __attribute__((aligned(16))) uint16_t sB[kBN][kBK + kPad];
    __shared__ float s_invt[kBM];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int v0 = blockIdx.x * kBN, m0 = blockIdx.y * kBM;
    if (tid < kBM && m0 + tid < M) s_invt[tid] = row_inv_temperature(temperature, m0 + tid, n);
    const int wm = wave >> 1, wn = wave & 1;
    const uint16_t* Wg = reinterpret_cast<const uint16_t*>(W);
    const uint16_t* Hg = reinterpret_cast<const uint16_t*>(H);

    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    // each thread moves two 16-byte pieces of each operand per k-block: piece q -> row q/8, k-offset (q%8)*8
    u32x4 ra[2], rb[2];
    auto fetch = [&](int kb) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int q = tid + t * kBlock, row = q >> 3, k = kb * kBK + (q & 7) * 8;
            const u32x4 zero = {0u, 0u, 0u, 0u};
            ra[t] = (m0 + row < M && k < d) ? *reinterpret_cast<const u32x4*>(Hg + (size_t)(m0 + row) * d + k) : zero;
            rb[t] = (v0 + row < V && k < d) ? *reinterpret_cast<const u32x4*>(Wg + (size_t)(v0 + row) * d + k) : zero;
        }
    };
    const int KB = (d + kBK - 1) / kBK;
    fetch(0);
    for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int q = tid + t * kBlock, row = q >> 3, kk = (q & 7) * 8;
            *reinterpret_cast<u32x4*>(&sA[row][kk]) = ra[t];
            *reinterpret_cast<u32x4*>(&sB[row][kk]) = rb[t];
        }
        __syncthreads();
        if (kb + 1 < KB) fetch(kb + 1);
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            const int kk = ks * 16 + 8 * (lane >> 5);
            const bf16x8 av = *reinterpret_cast<const bf16x8*>(&sA[wm * 32 + (lane & 31)][kk]);
            const bf16x8 bv = *reinterpret_cast<const bf16x8*>(&sB[wn * 32 + (lane & 31)][kk]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    store_tile_32x32(acc, m0 + wm * 32, v0 + wn * 32, M, V, NT, s_invt, m0, L, pm, ps);
}

// Workgroup barrier that orders LDS traffic only: it waits for this wave's LDS operations and nothing else, so
// a wave reaches it with its W requests still in flight.  (A barrier written so that it also waits for vector
// memory would stall a workgroup until all of its outstanding W requests have landed.)
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---------------------------------------------------------------- bf16, skinny M (<= 64 rows): W-streaming kernel
// With n*B <= 64 rows the GEMM moves 2*d bytes of W per n*B*2*d flops: it is bound by streaming W from HBM
// once, not by the matrix cores.  Design:
//   * 8 waves per workgroup, one workgroup per compute unit.  All of H (<= 64 x d bf16) is staged once into
//     LDS (rows padded by 16 bytes, so the 16-byte operand reads of 16 consecutive rows hit distinct banks).
//   * A pair of waves owns one 32-row vocabulary tile; each wave of the pair takes one half of K and streams
//     it k-block by k-block (32 rows x 128 bytes, coalesced 16-byte loads: 8 lanes cover one row's 128 bytes),
//     three k-blocks ahead of the one being multiplied.  W is read exactly once; no wave shares W with another.
//   * The MFMA wants "lane = vocabulary row, 8 consecutive k": each k-block goes through a wave-private
//     32 x 144-byte LDS patch that only re-maps lanes (write coalesced layout, read operand layout); LDS ops of
//     one wave execute in order, so the patch needs no barrier.
//   * W is the MFMA's row operand, so the accumulator is [vocabulary][result row]: the softmax partials of a
//     row are an in-register reduction plus one half-wave exchange.
//   * The two K-halves meet through the same patches (LDS-only barriers), each wave finishing one 32-row
//     block of the 64 x 32 result: logits (turned through the patch once more, stored as whole 128-byte lines
//     past L2) + softmax partials of the tile.
// KH = k-blocks (of 64) per wave = d / 128; MT = 32-row blocks of M (1 or 2).
constexpr int kSkinnyWaves = 8;
constexpr int kSkinnyThreads = kSkinnyWaves * 64;
constexpr int kPatchBytes = 32 * 144;

// ---------------------------------------------------------------- fused sampler (Alg. 1 lines 6-7 in the LM head's tail)
// A separate sampler kernel costs a launch gap and a cold start per draft position for half a megabyte of input.
// Instead every LM-head workgroup also publishes, per row, the (max, sum of exp) of each group of four tiles it
// finishes (128 vocabulary entries), waits for its stores, and bumps an arrival counter; the workgroup whose
// arrival completes the launch runs the sampler for every sampling row:
//   A  the group summaries of all rows ([NG][64] x 8 bytes) are staged in LDS (the H tiles are no longer needed);
//      per row: log-sum-exp over the groups (fixed order: 512 threads = rows x slices, slices combined in order);
//   B  per sequence (one wave each): group masses of the mixture  M_g = sum_j (w_j / S_j) s_jg exp(m_jg - m_j),
//      prefix over the groups in vocabulary order, the group where it crosses u * Z;
//   C  the 128 logits of that group for the sequence's n rows (written by another workgroup of this launch:
//      device-scope loads), the mixture's value at each, prefix, the token where it crosses, q(y), margin flags.
// Greedy rows need an arg-max over the whole vocabulary: they are left to the kernel that follows, unless the
// caller announced that none is expected -- then a greedy row is walked here by one wave, correct but slow.
struct TailArgs {
    int B, gamma, pos, NG;
    int greedy_here;           // 1: no arg-max kernel follows this launch
    uint64_t seed, round;
    const float* weights;
    const float* u_draft;
    double* draft_lse;
    int32_t* draft_tokens;
    float* draft_q;
    uint8_t* flags;
    unsigned long long* gsum;  // [NG][64]: low word = max, high word = sum of exp(. - max), as float bits
    uint32_t* ticket;          // nullptr: no fused sampler in this launch
};

constexpr int kTailLoads = 32;                      // staged 8-byte entries per thread and batch

// Bytes of dynamic LDS the tail needs for NG groups and MP (32 or 64) table rows.
static size_t tail_lds_bytes(int NG, int MP) {
    return (size_t)NG * (MP + 1) * 8;
}

// Called by threads tid < 64 of a workgroup once the partials of the group's four tiles are in s_pstage.
__device__ __forceinline__ void publish_group_summary(const TailArgs& t, const float* s_pstage, int row, int M, int g,
                                                      int NT) {
    if (row >= M) return;
    const float* pmr = s_pstage + (0 * 64 + row) * 4;
    const float* psr = s_pstage + (1 * 64 + row) * 4;
    float gm = -INFINITY;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (g * 4 + q < NT) gm = fmaxf(gm, pmr[q]);
    float gs = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (g * 4 + q < NT && psr[q] > 0.f) gs += psr[q] * __expf(pmr[q] - gm);
    const unsigned long long packed =
        (unsigned long long)__builtin_bit_cast(uint32_t, gm) | ((unsigned long long)__builtin_bit_cast(uint32_t, gs) << 32);
    __hip_atomic_store(&t.gsum[(size_t)g * 64 + row], packed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int MP>
__device__ __forceinline__ void sampler_tail(const TailArgs& t, int M, int V, int n, const float* __restrict__ temperature,
                                          const float* L, unsigned char* lds) {
    constexpr int SL = kSkinnyThreads / MP;         // slices of the group range per row
    constexpr int RP = MP + 1;                      // padded row count: lane-to-lane stride of 2 banks
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int NG = t.NG;
    float2* sg = reinterpret_cast<float2*>(lds);                                     // [NG][RP]
    __shared__ float s_redm[SL * MP];
    __shared__ double s_reds[SL * MP];
    __shared__ double s_S[64], s_c[64];                                              // s_c = w_j / S_j
    __shared__ float s_m[64];

    // ---- A: stage every row's group summaries (device-scope loads, kTailLoads in flight per thread; the loads
    //      are never predicated -- an index past the end is clamped -- so that none of them waits for another)
    const int total = NG * MP;
    for (int base = 0; base < total; base += kTailLoads * kSkinnyThreads) {
        unsigned long long v[kTailLoads];
#pragma unroll
        for (int k = 0; k < kTailLoads; ++k) {
            const int idx = min(base + k * kSkinnyThreads + tid, total - 1);
            v[k] = __hip_atomic_load(&t.gsum[(size_t)(idx / MP) * 64 + (idx % MP)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int k = 0; k < kTailLoads; ++k) {
            const int idx = base + k * kSkinnyThreads + tid;
            if (idx < total)
                sg[(idx / MP) * RP + (idx % MP)] = make_float2(__builtin_bit_cast(float, (uint32_t)v[k]),
                                                               __builtin_bit_cast(float, (uint32_t)(v[k] >> 32)));
        }
    }
    __syncthreads();
    {
        const int row = tid % MP, slice = tid / MP;
        const bool rlive = row < M;
        float ml = -INFINITY;
        if (rlive)
            for (int g = slice; g < NG; g += SL) ml = fmaxf(ml, sg[g * RP + row].x);
        s_redm[slice * MP + row] = ml;
        __syncthreads();
        float m = -INFINITY;
#pragma unroll
        for (int q = 0; q < SL; ++q) m = fmaxf(m, s_redm[q * MP + row]);
        float sl = 0.f;
        if (rlive)
            for (int g = slice; g < NG; g += SL) {
                const float2 e = sg[g * RP + row];
                if (e.y > 0.f) sl += e.y * __expf(e.x - m);
            }
        s_reds[slice * MP + row] = (double)sl;
        __syncthreads();
        if (tid < M) {                              // tid < MP here, so row == tid and m is this row's maximum
            double S = 0.0;
#pragma unroll
            for (int q = 0; q < SL; ++q) S += s_reds[q * MP + tid];
            const int b = tid / n, j = tid % n;
            s_m[tid] = m;
            s_S[tid] = S;
            s_c[tid] = (double)t.weights[(size_t)b * n + j] / S;
            t.draft_lse[((size_t)t.pos * t.B + b) * n + j] = (double)m + log(S);
        }
        __syncthreads();
    }

    // ---- B + C: one wave per sequence
    for (int b = wave; b < t.B; b += kSkinnyWaves) {
        const float T = temperature[b];
        const bool greedy = !(T > 0.f);
        const float invT = greedy ? 1.f : 1.f / T;
        const size_t out_idx = (size_t)b * t.gamma + t.pos;
        const int r0 = b * n;
        const float* rows = L + (size_t)r0 * V;
        if (greedy) {
            if (!t.greedy_here) continue;           // the arg-max kernel that follows decides this row
            Top2 best = top2_empty();
            for (int v0 = 0; v0 < V; v0 += 4 * kWave) {
                float q[4] = {0.f, 0.f, 0.f, 0.f};
                for (int j = 0; j < n; ++j) {
                    const float cj = (float)s_c[r0 + j], mj = s_m[r0 + j];
                    float x[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = v0 + e * kWave + lane;
                        x[e] = (v < V) ? published_load(rows + (size_t)j * V + v) : -INFINITY;
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) q[e] += cj * __expf(x[e] * invT - mj);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int v = v0 + e * kWave + lane;
                    if (v < V) best = top2_push(best, q[e], v);
                }
            }
            best = wave_top2(best);
            if (lane == 0) {
                const int y = (best.i1 >= 0 && best.i1 < V) ? best.i1 : 0;
                double f = 0.0;
                for (int j = 0; j < n; ++j)
                    f += s_c[r0 + j] * (double)__expf(published_load(rows + (size_t)j * V + y) * invT - s_m[r0 + j]);
                uint32_t flag = 0;
                if (V > 1 && (best.v1 - best.v2) < kMargin * fabsf(best.v1)) flag |= TABED_FLAG_SAMPLE_MARGIN;
                t.draft_tokens[out_idx] = y;
                t.draft_q[out_idx] = (float)f;
                t.flags[out_idx] = (uint8_t)flag;
            }
            continue;
        }
        const float u = t.u_draft ? t.u_draft[out_idx] : tabed_uniform(t.seed, t.round, (uint32_t)b, (uint32_t)t.pos, 0);
        double Z = 0.0;
        for (int j = 0; j < n; ++j) Z += s_c[r0 + j] * s_S[r0 + j];
        const double target = (double)u * Z;
        // group masses, 64 groups per sweep (lane = group: neighbouring lanes are 2 banks apart), running prefix
        double carry = 0.0, P = 0.0, Plast = 0.0;
        int gstar = -1, glast = -1;
        for (int g0 = 0; g0 < NG; g0 += kWave) {
            const int g = g0 + lane;
            double mass = 0.0;
            if (g < NG)
                for (int j = 0; j < n; ++j) {
                    const float2 e = sg[g * RP + r0 + j];
                    if (e.y > 0.f) mass += s_c[r0 + j] * (double)(e.y * __expf(e.x - s_m[r0 + j]));
                }
            const double cdf = carry + wave_inclusive_scan(mass);
            const unsigned long long cross = __ballot(mass > 0.0 && cdf > target);
            const unsigned long long live = __ballot(mass > 0.0);
            if (gstar < 0 && cross) {
                const int l = __ffsll((long long)cross) - 1;
                gstar = g0 + l;
                P = lane_f64(cdf - mass, l);
            }
            if (live) {
                const int l = 63 - __clzll((long long)live);
                glast = g0 + l;
                Plast = lane_f64(cdf - mass, l);
            }
            carry = lane_f64(cdf, 63);
            if (gstar >= 0) break;                  // uniform over the wave
        }
        if (gstar < 0) { gstar = glast; P = Plast; }   // rounding let nothing cross: the last group with mass
        if (gstar < 0) {                               // every mass is zero
            if (lane == 0) {
                t.draft_tokens[out_idx] = 0;
                t.draft_q[out_idx] = 0.f;
                t.flags[out_idx] = (uint8_t)(TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE);
            }
            continue;
        }
        // the group's 128 logits of every draft row: all loads first (at most 2 x 16), then the mixture
        float x[2][TABED_MAX_N];
#pragma unroll
        for (int j = 0; j < TABED_MAX_N; ++j)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {          // unpredicated: row and column clamped, masked below
                const int v = min(gstar * 128 + hh * kWave + lane, V - 1);
                x[hh][j] = published_load(rows + (size_t)min(j, n - 1) * V + v);
            }
        double f[2] = {0.0, 0.0};
#pragma unroll
        for (int j = 0; j < TABED_MAX_N; ++j)
            if (j < n) {
                const double cj = s_c[r0 + j];
                const float mj = s_m[r0 + j];
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
                    if (gstar * 128 + hh * kWave + lane < V) f[hh] += cj * (double)__expf(x[hh][j] * invT - mj);
            }
        const double inc0 = wave_inclusive_scan(f[0]);
        const double inc1 = lane_f64(inc0, 63) + wave_inclusive_scan(f[1]);
        const double cdf[2] = {P + inc0, P + inc1};
        const unsigned long long cross0 = __ballot(cdf[0] > target && f[0] > 0.0), cross1 = __ballot(cdf[1] > target && f[1] > 0.0);
        const unsigned long long live0 = __ballot(f[0] > 0.0), live1 = __ballot(f[1] > 0.0);
        int ph, pl;                                  // half and lane of the chosen entry
        uint32_t flag = 0;
        if (cross0) { ph = 0; pl = __ffsll((long long)cross0) - 1; }
        else if (cross1) { ph = 1; pl = __ffsll((long long)cross1) - 1; }
        else {
            flag = TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE;
            if (live1) { ph = 1; pl = 63 - __clzll((long long)live1); }
            else if (live0) { ph = 0; pl = 63 - __clzll((long long)live0); }
            else { ph = 0; pl = 0; }
        }
        if (lane == pl) {
            const int v = gstar * 128 + ph * kWave + lane;
            const double fv = ph ? f[1] : f[0], cv = ph ? cdf[1] : cdf[0];
            const double tol = (double)kMargin * Z;
            if (fabs(cv - target) < tol && v + 1 < V) flag |= TABED_FLAG_SAMPLE_MARGIN;
            if (v > 0 && fabs((cv - fv) - target) < tol) flag |= TABED_FLAG_SAMPLE_MARGIN;
            t.draft_tokens[out_idx] = v < V ? v : V - 1;
            t.draft_q[out_idx] = (float)fv;
            t.flags[out_idx] = (uint8_t)flag;
        }
    }
}

template <int KH, int MT, bool FUSE>
__global__ __launch_bounds__(kSkinnyThreads) void k_lmhead_skinny(int M, int V, int n, int NT, int num_tiles,
                                                                  const uint16_t* __restrict__ W,
                                                                  const uint16_t* __restrict__ H,
                                                                  const float* __restrict__ temperature,
                                                                  float* L, float* __restrict__ pm,
                                                                  float* __restrict__ ps, TailArgs tail) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ float s_invt[64];
    __shared__ __attribute__((aligned(16))) float s_pstage[2 * 64 * 4];   // softmax partials of the group's 4 tiles
    constexpr int d = KH * 128;
    constexpr int CH = d / 8;                       // 16-byte chunks per row of H / W
    constexpr int HROW = CH * 16 + 16;              // padded LDS row of H in bytes
    unsigned char* const ldsH = lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pair = wave & 3, khalf = wave >> 2;
    unsigned char* const patch = lds + MT * 32 * HROW + wave * kPatchBytes;
    unsigned char* const partner_patch = lds + MT * 32 * HROW + (wave ^ 4) * kPatchBytes;
    const int nn = lane & 31, half = lane >> 5;
    if (tid < M) s_invt[tid] = row_inv_temperature(temperature, tid, n);

    // ---- request H first (it must land before any MFMA)
    u32x4 hreg[MT * KH];
#pragma unroll
    for (int q = 0; q < MT * KH; ++q) {
        // rows >= M are clamped, not zeroed: their results are never stored
        const int p = tid + q * kSkinnyThreads, row = min(p / CH, M - 1), c = p % CH;
        hreg[q] = *reinterpret_cast<const u32x4*>(H + (size_t)row * d + c * 8);
    }
    const int lrow = lane >> 3, lchunk = lane & 7;  // coalesced load layout: instruction i covers rows 8i..8i+7
    u32x4 wreg[KH][4];
    // Requests of one k-block (4 coalesced 16-byte loads per lane).  Vocabulary rows >= V (ragged last tile,
    // idle pair of the last group) are clamped to row V-1: the epilogue masks them, so no load is predicated.
    // (element offsets from W, not pointers: a pointer carried in an array degrades to a flat address and
    // flat loads also count as LDS traffic, which would stall every LDS read behind them)
    auto aim_tile = [&](size_t (&off)[4], int tile) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = min(tile * 32 + 8 * i + lrow, V - 1);
            off[i] = (size_t)v * d + (size_t)khalf * (KH * 64) + lchunk * 8;
        }
    };
    auto request_kblock = [&](const size_t (&off)[4], int kb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) wreg[kb][i] = *reinterpret_cast<const u32x4*>(W + off[i] + kb * 64);
    };
    // Only the first kPF k-blocks of W are requested before H has landed.  Measured on MI355X: a compute unit
    // accepts a bounded number of outstanding requests, so issuing a whole half-tile takes about as long as
    // streaming it, and with all of W queued behind them the H loads came back ~5 us late (nothing can start
    // without H).  With kPF k-blocks queued H lands at ~1.7 us and the first W data follows at once; the rest
    // of W is requested k-block by k-block, kPF ahead of the one being multiplied.
    constexpr int kPF = (KH < 3) ? KH : 3;
    size_t src[4];                                 // the tile whose k-blocks are being requested
    aim_tile(src, blockIdx.x * 4 + pair);
#pragma unroll
    for (int kb = 0; kb < kPF; ++kb) request_kblock(src, kb);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < MT * KH; ++q) {
        const int p = tid + q * kSkinnyThreads, row = p / CH, c = p % CH;
        *reinterpret_cast<u32x4*>(ldsH + row * HROW + c * 16) = hreg[q];
    }
    lds_barrier();                                 // also publishes s_invt

    for (int g = blockIdx.x;; g += gridDim.x) {    // tile group g = 4 tiles, one per wave pair; trip count is
        const int this_tile = g * 4 + pair;        // uniform over the workgroup (barriers inside)
        f32x16 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
        const bool more = ((g + (int)gridDim.x) * 4 < num_tiles);   // this workgroup has another tile group
        size_t nsrc[4];
        aim_tile(nsrc, more ? this_tile + (int)gridDim.x * 4 : this_tile);
#pragma unroll
        for (int kb = 0; kb < KH; ++kb) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *reinterpret_cast<u32x4*>(patch + (8 * i + lrow) * 144 + lchunk * 16) = wreg[kb][i];
            // the registers of k-block kb are free again: request the k-block kPF ahead (of this tile, or of
            // the workgroup's next tile once this one is fully requested)
            __builtin_amdgcn_sched_barrier(0);
            if (kb + kPF < KH) request_kblock(src, kb + kPF);
            else if (more) request_kblock(nsrc, kb + kPF - KH);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 bv = *reinterpret_cast<const bf16x8*>(patch + nn * 144 + (2 * ks + half) * 16);
                const int hc = (khalf * KH + kb) * 8 + 2 * ks + half;       // chunk index inside H's row
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const bf16x8 av = *reinterpret_cast<const bf16x8*>(ldsH + (mt * 32 + nn) * HROW + hc * 16);
                    // W fragment as the row operand: the accumulator comes out as [vocabulary][result row]
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv, av, acc[mt], 0, 0, 0);
                }
            }
        }

        // ---- the two K-halves meet: each wave hands the partner the 32-row block the partner finishes
        //      (MT == 2: wave khalf finishes block khalf; MT == 1: the khalf == 0 wave finishes block 0)
        f32x16 fin = acc[0], giv = acc[MT - 1];
        if (MT == 2 && khalf == 1) { fin = acc[MT - 1]; giv = acc[0]; }
        if (MT == 2 || khalf == 1) {
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<float4*>(patch + g * 1024 + lane * 16) =
                    make_float4(giv[4 * g], giv[4 * g + 1], giv[4 * g + 2], giv[4 * g + 3]);
        }
        lds_barrier();
        if (MT == 2 || khalf == 0) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 o = *reinterpret_cast<const float4*>(partner_patch + g * 1024 + lane * 16);
                fin[4 * g] += o.x; fin[4 * g + 1] += o.y; fin[4 * g + 2] += o.z; fin[4 * g + 3] += o.w;
            }
        }
        lds_barrier();                                 // both patches of the pair are read: they may be reused
        if ((MT == 2 || khalf == 0) && this_tile < num_tiles)
            store_tile_32x32_t<FUSE>(fin, (MT == 2) ? khalf * 32 : 0, this_tile * 32, M, V, NT, s_invt, L, pm, ps, patch, s_pstage, pair);
        // the four tiles of this group sit side by side in a row of the partial tables: 16 bytes per row
        lds_barrier();
        if (tid < 128 && (tid & 63) < M) {
            const int arr = tid >> 6, row = tid & 63, t0 = g * 4;
            float* dst = (arr == 0 ? pm : ps) + (size_t)row * NT + t0;
            const float* srcp = s_pstage + (arr * 64 + row) * 4;
            if ((NT & 3) == 0 && t0 + 3 < NT) *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(srcp);
            else for (int q = 0; q < 4; ++q) if (t0 + q < NT) dst[q] = srcp[q];
        }
        if (FUSE && tid >= 128 && tid < 192) publish_group_summary(tail, s_pstage, tid - 128, M, g, NT);
        if (!more) break;
#pragma unroll
        for (int i = 0; i < 4; ++i) src[i] = nsrc[i];
    }
    if (FUSE) {
        // every store of this workgroup (logits, group summaries) is acknowledged before its arrival counts
        __shared__ int s_last;
        publish_barrier();
        if (tid == 0) s_last = arrive(tail.ticket, gridDim.x) ? 1 : 0;
        __syncthreads();
        if (s_last) sampler_tail<MT * 32>(tail, M, V, n, temperature, L, lds);
    }
}

// ---------------------------------------------------------------- bf16, skinny M, larger hidden sizes
// Same design as k_lmhead_skinny for hidden sizes whose H (64 x d) does not fit LDS: K is walked in chunks of
// KH*128, and LDS holds one chunk of H at a time.  The next chunk of H is requested into registers at the
// start of a chunk's k-loop and written to LDS between two LDS-only barriers at its end; the W request
// stream (kPF k-blocks ahead) runs straight across chunk boundaries.  d = nchunks * KH * 128.
template <int KH, int MT, bool FUSE>
__global__ __launch_bounds__(kSkinnyThreads) void k_lmhead_skinny_kc(int M, int V, int n, int NT, int num_tiles,
                                                                     int nchunks,
                                                                     const uint16_t* __restrict__ W,
                                                                     const uint16_t* __restrict__ H,
                                                                     const float* __restrict__ temperature,
                                                                     float* L, float* __restrict__ pm,
                                                                     float* __restrict__ ps, TailArgs tail) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ float s_invt[64];
    __shared__ __attribute__((aligned(16))) float s_pstage[2 * 64 * 4];   // softmax partials of the group's 4 tiles
    constexpr int DC = KH * 128;                    // k per chunk
    constexpr int CH = DC / 8;                      // 16-byte pieces per row of one H chunk
    constexpr int HROW = CH * 16 + 16;              // padded LDS row of H in bytes
    const int d = nchunks * DC;
    unsigned char* const ldsH = lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pair = wave & 3, khalf = wave >> 2;
    unsigned char* const patch = lds + MT * 32 * HROW + wave * kPatchBytes;
    unsigned char* const partner_patch = lds + MT * 32 * HROW + (wave ^ 4) * kPatchBytes;
    const int nn = lane & 31, half = lane >> 5;
    if (tid < M) s_invt[tid] = row_inv_temperature(temperature, tid, n);

    u32x4 hreg[MT * KH];
    auto request_h = [&](int chunk) {               // rows >= M are clamped: their results are never stored
#pragma unroll
        for (int q = 0; q < MT * KH; ++q) {
            const int p = tid + q * kSkinnyThreads, row = min(p / CH, M - 1), c = p % CH;
            hreg[q] = *reinterpret_cast<const u32x4*>(H + (size_t)row * d + (size_t)chunk * DC + c * 8);
        }
    };
    auto write_h = [&]() {
#pragma unroll
        for (int q = 0; q < MT * KH; ++q) {
            const int p = tid + q * kSkinnyThreads, row = p / CH, c = p % CH;
            *reinterpret_cast<u32x4*>(ldsH + row * HROW + c * 16) = hreg[q];
        }
    };
    const int lrow = lane >> 3, lchunk = lane & 7;
    u32x4 wreg[KH][4];
    auto aim_tile = [&](size_t (&off)[4], int tile) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = min(tile * 32 + 8 * i + lrow, V - 1);
            off[i] = (size_t)v * d + (size_t)khalf * (KH * 64) + lchunk * 8;
        }
    };
    auto request_kblock = [&](const size_t (&off)[4], int chunk, int kb) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            wreg[kb][i] = *reinterpret_cast<const u32x4*>(W + off[i] + (size_t)chunk * DC + kb * 64);
    };
    constexpr int kPF = 3;                          // KH >= 4 here
    request_h(0);
    size_t src[4];
    aim_tile(src, blockIdx.x * 4 + pair);
#pragma unroll
    for (int kb = 0; kb < kPF; ++kb) request_kblock(src, 0, kb);
    __builtin_amdgcn_sched_barrier(0);
    write_h();
    lds_barrier();                                  // also publishes s_invt

    for (int g = blockIdx.x;; g += gridDim.x) {
        const int this_tile = g * 4 + pair;
        f32x16 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
        const bool more = ((g + (int)gridDim.x) * 4 < num_tiles);
        size_t nsrc[4];
        aim_tile(nsrc, more ? this_tile + (int)gridDim.x * 4 : this_tile);
        for (int chunk = 0; chunk < nchunks; ++chunk) {
            const bool last_chunk = (chunk + 1 == nchunks);
            const bool h_next = !last_chunk || more;  // another chunk of H follows (of this tile or the next)
            if (h_next) request_h(last_chunk ? 0 : chunk + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kb = 0; kb < KH; ++kb) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    *reinterpret_cast<u32x4*>(patch + (8 * i + lrow) * 144 + lchunk * 16) = wreg[kb][i];
                __builtin_amdgcn_sched_barrier(0);
                if (kb + kPF < KH) request_kblock(src, chunk, kb + kPF);
                else if (!last_chunk) request_kblock(src, chunk + 1, kb + kPF - KH);
                else if (more) request_kblock(nsrc, 0, kb + kPF - KH);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const bf16x8 bv = *reinterpret_cast<const bf16x8*>(patch + nn * 144 + (2 * ks + half) * 16);
                    const int hc = (khalf * KH + kb) * 8 + 2 * ks + half;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const bf16x8 av = *reinterpret_cast<const bf16x8*>(ldsH + (mt * 32 + nn) * HROW + hc * 16);
                        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv, av, acc[mt], 0, 0, 0);
                    }
                }
            }
            if (h_next) {
                lds_barrier();                      // every wave is done with this chunk of H
                write_h();
                lds_barrier();
            }
        }

        f32x16 fin = acc[0], giv = acc[MT - 1];
        if (MT == 2 && khalf == 1) { fin = acc[MT - 1]; giv = acc[0]; }
        if (MT == 2 || khalf == 1) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<float4*>(patch + q * 1024 + lane * 16) =
                    make_float4(giv[4 * q], giv[4 * q + 1], giv[4 * q + 2], giv[4 * q + 3]);
        }
        lds_barrier();
        if (MT == 2 || khalf == 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 o = *reinterpret_cast<const float4*>(partner_patch + q * 1024 + lane * 16);
                fin[4 * q] += o.x; fin[4 * q + 1] += o.y; fin[4 * q + 2] += o.z; fin[4 * q + 3] += o.w;
            }
        }
        lds_barrier();
        if ((MT == 2 || khalf == 0) && this_tile < num_tiles)
            store_tile_32x32_t<FUSE>(fin, (MT == 2) ? khalf * 32 : 0, this_tile * 32, M, V, NT, s_invt, L, pm, ps, patch, s_pstage, pair);
        // the four tiles of this group sit side by side in a row of the partial tables: 16 bytes per row
        lds_barrier();
        if (tid < 128 && (tid & 63) < M) {
            const int arr = tid >> 6, row = tid & 63, t0 = g * 4;
            float* dst = (arr == 0 ? pm : ps) + (size_t)row * NT + t0;
            const float* srcp = s_pstage + (arr * 64 + row) * 4;
            if ((NT & 3) == 0 && t0 + 3 < NT) *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(srcp);
            else for (int q = 0; q < 4; ++q) if (t0 + q < NT) dst[q] = srcp[q];
        }
        if (FUSE && tid >= 128 && tid < 192) publish_group_summary(tail, s_pstage, tid - 128, M, g, NT);
        if (!more) break;
#pragma unroll
        for (int i = 0; i < 4; ++i) src[i] = nsrc[i];
    }
    if (FUSE) {
        // every store of this workgroup (logits, group summaries) is acknowledged before its arrival counts
        __shared__ int s_last;
        publish_barrier();
        if (tid == 0) s_last = arrive(tail.ticket, gridDim.x) ? 1 : 0;
        __syncthreads();
        if (s_last) sampler_tail<MT * 32>(tail, M, V, n, temperature, L, lds);
    }
}

// ---------------------------------------------------------------- bf16, many rows (M > 64): MFMA-bound tiled GEMM
// With hundreds of rows (stress shape: n*B = 512) the LM head is a real GEMM: 2*M*d*V flops against one
// pass over W.  Workgroup tile 256 (rows) x 256 (vocabulary) x 32 (k), 8 waves, each wave a 128 (rows) x 64
// (vocabulary) block (2 x 4 MFMA 32x32x16 tiles, W as the row operand so the accumulator is
// [vocabulary][row] and the cheap transposed epilogue applies).  Both operands are staged through LDS in two
// buffers; the operand fragments of k-step s+1 are read from LDS while the MFMAs of k-step s run, and the
// global loads of k-blocks i+2 and i+3 are in flight (two register sets) while k-block i is multiplied --
// one barrier per k-block.  Rows padded by 16 bytes against bank conflicts.  Workgroups are numbered so that
// the row blocks that share a vocabulary block run back to back on the same XCD (workgroup w goes to XCD
// w % 8): W is then read from HBM once and from L2 afterwards.
constexpr int kLBM = 256, kLBN = 256, kLBK = 32, kLRow = (kLBK + 8) * 2;   // LDS row stride in bytes (80)
constexpr int kLCh = kLBK / 8;                                              // 16-byte chunks per row of a k-block
constexpr int kLargeStage = (kLBM + kLBN) * kLRow;                          // bytes per buffer (40960)

// NW = waves per workgroup: 8 (each wave 128 rows x 64 vocabulary entries, two waves per SIMD) or 4 (each wave
// 128 x 128, one wave per SIMD with the accumulators in the upper half of the register file).
constexpr int kLargeWaves = 8;

template <int NW>
__global__ __launch_bounds__(NW * 64) void k_lmhead_large(int M, int d, int V, int n, int NT, int mblocks,
                                                                const uint16_t* __restrict__ W,
                                                                const uint16_t* __restrict__ H,
                                                                const float* __restrict__ temperature,
                                                                float* __restrict__ L, float* __restrict__ pm,
                                                                float* __restrict__ ps) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ float s_invt[kLBM];
    constexpr int kLargeThreads = NW * 64;
    constexpr int kLWPieces = kLBN * kLCh / kLargeThreads, kLHPieces = kLBM * kLCh / kLargeThreads;
    static_assert(kLBN * kLCh % kLargeThreads == 0 && kLBM * kLCh % kLargeThreads == 0, "staging split");
    constexpr int WNT = (NW == 8) ? 2 : 4;                // 32-wide vocabulary tiles per wave
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nn = lane & 31, half = lane >> 5;
    // XCD-aware numbering: workgroup w runs on XCD w % 8; consecutive slots of one XCD walk the row blocks
    // of one vocabulary block before moving to the next vocabulary block.
    const int w = blockIdx.x, xcd = w & 7, slot = w >> 3;
    const int mb = slot % mblocks, nb = (slot / mblocks) * 8 + xcd;
    const int m0 = mb * kLBM, v0 = nb * kLBN;
    if (v0 >= V) return;                                  // uniform: padding workgroups of the last XCD round
    const int wm = (NW == 8) ? wave >> 2 : wave >> 1;     // wave block: rows m0 + 128*wm ..,
    const int wn = (NW == 8) ? wave & 3 : wave & 1;       // vocabulary v0 + 32*WNT*wn ..
    if (tid < kLBM && m0 + tid < M) s_invt[tid] = row_inv_temperature(temperature, m0 + tid, n);

    // ---- global -> register staging: two register sets, so that the loads of k-block kb+2 and kb+3 are in
    //      flight while k-block kb is multiplied (one k-block is only ~1000 cycles of MFMA work per SIMD,
    //      less than an L2 round trip).  kLWPieces of W and kLHPieces of H per thread and set (16 bytes each).
    u32x4 rw[2][kLWPieces], rh[2][kLHPieces];
    auto fetch = [&](int kb, auto set_c) {
        constexpr int S = decltype(set_c)::value;
        const int k = kb * kLBK;
#pragma unroll
        for (int t = 0; t < kLWPieces; ++t) {
            const int q = tid + t * kLargeThreads, row = q / kLCh, c = q % kLCh;
            const int v = min(v0 + row, V - 1);           // clamped rows are masked in the epilogue
            rw[S][t] = *reinterpret_cast<const u32x4*>(W + (size_t)v * d + k + c * 8);
        }
#pragma unroll
        for (int t = 0; t < kLHPieces; ++t) {
            const int q = tid + t * kLargeThreads, row = q / kLCh, c = q % kLCh;
            const int m = min(m0 + row, M - 1);
            rh[S][t] = *reinterpret_cast<const u32x4*>(H + (size_t)m * d + k + c * 8);
        }
    };
    auto stash = [&](int buf, auto set_c) {
        constexpr int S = decltype(set_c)::value;
        unsigned char* sW = lds + buf * kLargeStage;
        unsigned char* sH = sW + kLBN * kLRow;
#pragma unroll
        for (int t = 0; t < kLWPieces; ++t) {
            const int q = tid + t * kLargeThreads, row = q / kLCh, c = q % kLCh;
            *reinterpret_cast<u32x4*>(sW + row * kLRow + c * 16) = rw[S][t];
        }
#pragma unroll
        for (int t = 0; t < kLHPieces; ++t) {
            const int q = tid + t * kLargeThreads, row = q / kLCh, c = q % kLCh;
            *reinterpret_cast<u32x4*>(sH + row * kLRow + c * 16) = rh[S][t];
        }
    };
    using Set0 = std::integral_constant<int, 0>;
    using Set1 = std::integral_constant<int, 1>;

    f32x16 acc[WNT][4];                                   // [vocabulary tile][row tile]
#pragma unroll
    for (int a = 0; a < WNT; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    auto multiply = [&](int buf) {
        const unsigned char* sW = lds + buf * kLargeStage;
        const unsigned char* sH = sW + kLBN * kLRow;
        // operand fragments of k-step ks+1 are read from LDS while the MFMAs of k-step ks run
        bf16x8 wf[2][WNT], hf[2][4];
        auto read_frags = [&](int ks, int set) {
#pragma unroll
            for (int a = 0; a < WNT; ++a)
                wf[set][a] = *reinterpret_cast<const bf16x8*>(sW + (wn * 32 * WNT + a * 32 + nn) * kLRow + (2 * ks + half) * 16);
#pragma unroll
            for (int b = 0; b < 4; ++b)
                hf[set][b] = *reinterpret_cast<const bf16x8*>(sH + (wm * 128 + b * 32 + nn) * kLRow + (2 * ks + half) * 16);
        };
        read_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < kLBK / 16; ++ks) {
            if (ks + 1 < kLBK / 16) read_frags(ks + 1, (ks + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);            // keep the reads ahead of the MFMAs they overlap with
#pragma unroll
            for (int a = 0; a < WNT; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks & 1][a], hf[ks & 1][b], acc[a][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // k-block j lives in register set j & 1 until it is written to LDS buffer j & 1.  KB is even (d % 64 == 0).
    const int KB = d / kLBK;
    fetch(0, Set0{});
    stash(0, Set0{});
    fetch(1, Set1{});
    if (2 < KB) fetch(2, Set0{});
    lds_barrier();
    for (int kb = 0; kb < KB; kb += 2) {
        multiply(0);                                      // k-block kb
        if (kb + 1 < KB) stash(1, Set1{});                // k-block kb+1 (requested two iterations ago)
        if (kb + 3 < KB) fetch(kb + 3, Set1{});
        lds_barrier();
        if (kb + 1 < KB) multiply(1);                     // k-block kb+1
        if (kb + 2 < KB) stash(0, Set0{});                // k-block kb+2
        if (kb + 4 < KB) fetch(kb + 4, Set0{});
        lds_barrier();
    }
    // ---- epilogue: every wave turns its four 32x32 blocks through a private patch carved from buffer 0
    unsigned char* tpatch = lds + wave * kPatchBytes;
#pragma unroll
    for (int a = 0; a < WNT; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
            store_tile_32x32_t(acc[a][b], m0 + wm * 128 + b * 32, v0 + wn * 32 * WNT + a * 32, M, V, NT, s_invt - m0, L, pm, ps,
                               tpatch);
}

// ---------------------------------------------------------------- fp32 operands: one output per thread
// Workgroup = 8 rows x 32 vocabulary entries; a half-wave shares one row, so the tile partials are a
// half-wave reduction.  Only the tiny correctness configuration stores fp32 weights.
__global__ __launch_bounds__(kBlock) void k_lmhead_f32(int M, int d, int V, int n, int NT,
                                                       const float* __restrict__ W, const float* __restrict__ H,
                                                       const float* __restrict__ temperature,
                                                       float* __restrict__ L, float* __restrict__ pm,
                                                       float* __restrict__ ps) {
    const int tid = threadIdx.x;
    const int m = blockIdx.y * 8 + (tid >> 5);
    const int v = blockIdx.x * kTileV + (tid & 31);
    const bool live = (m < M);
    float s = -INFINITY;
    if (live && v < V) {
        const float* w = W + (size_t)v * d;
        const float* h = H + (size_t)m * d;
        double acc = 0.0;
        for (int k = 0; k < d; ++k) acc += (double)h[k] * (double)w[k];
        const float x = (float)acc;
        L[(size_t)m * V + v] = x;
        s = x * row_inv_temperature(temperature, m, n);
    }
    const float mx = half_max(s);
    const float e = (s > -INFINITY) ? __expf(s - mx) : 0.f;
    const float sum = half_sum(e);
    if (live && (tid & 31) == 0) {
        pm[(size_t)m * NT + blockIdx.x] = mx;
        ps[(size_t)m * NT + blockIdx.x] = sum;
    }
}

// Chunked variant: d a multiple of 768, 512 or 896 (k per chunk), at least two chunks.
static int skinny_kc_kh(const tabed_cfg& c, int M) {
    if (c.w_dtype != 1 || M > 64) return 0;
    // with two row blocks the 512-wide chunk is the one that keeps the H prefetch in registers without spills
    const int order_two[3] = {4, 6, 7}, order_one[3] = {6, 4, 7};
    for (int KH : (M > 32 ? order_two : order_one))
        if (c.d % (KH * 128) == 0 && c.d / (KH * 128) >= 2) return KH;
    return 0;
}

// Raises a kernel's dynamic-LDS limit once per process; a failure is remembered and returned by every later call.
template <typename K>
static hipError_t raise_lds_limit(K kernel, size_t lds, std::once_flag& once, hipError_t& rc) {
    std::call_once(once, [&] {
        rc = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    return rc;
}

static size_t skinny_lds_bytes(int KH, int MT) { return (size_t)MT * 32 * (KH * 256 + 16) + (size_t)kSkinnyWaves * kPatchBytes; }

// The fused sampler applies when the group summaries of every row fit the kernel's dynamic LDS, and the logits
// rows are 16-byte aligned (V % 4 == 0: the write-through stores are whole 16-byte pieces).
static bool tail_fits(const tabed_cfg& c, const WsLayout& Lay, int KH, int MT) {
    return c.V % 4 == 0 && (long long)Lay.M * c.V * 4 < (1ll << 31) &&
           tail_lds_bytes(Lay.NG, MT * 32) <= skinny_lds_bytes(KH, MT);
}

template <int KH, int MT, bool FUSE>
static hipError_t launch_skinny_kc_t(const ProfScope* prof, const tabed_cfg& c, const WsLayout& Lay, int M, const void* W,
                                     const void* H, const float* temperature, float* logits, float* pm, float* ps,
                                     const TailArgs& tail, hipStream_t s) {
    const size_t lds = skinny_lds_bytes(KH, MT);
    static std::once_flag attr_once;
    static hipError_t attr_rc = hipSuccess;
    if (raise_lds_limit(&k_lmhead_skinny_kc<KH, MT, FUSE>, lds, attr_once, attr_rc) != hipSuccess) return attr_rc;
    const int num_tiles = Lay.NT, groups = (num_tiles + 3) / 4;
    const dim3 grid(groups < 256 ? groups : 256);
    launch(prof, k_lmhead_skinny_kc<KH, MT, FUSE>, grid, dim3(kSkinnyThreads), lds, s, M, c.V, c.n, Lay.NT, num_tiles,
           c.d / (KH * 128), static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(H), temperature, logits, pm, ps,
           tail);
    return hipSuccess;
}

template <int KH, int MT, bool FUSE>
static hipError_t launch_skinny_t(const ProfScope* prof, const tabed_cfg& c, const WsLayout& Lay, int M, const void* W,
                                  const void* H, const float* temperature, float* logits, float* pm, float* ps,
                                  const TailArgs& tail, hipStream_t s) {
    const size_t lds = skinny_lds_bytes(KH, MT);
    static std::once_flag attr_once;                   // raise the dynamic-LDS limit of this instantiation once
    static hipError_t attr_rc = hipSuccess;
    if (raise_lds_limit(&k_lmhead_skinny<KH, MT, FUSE>, lds, attr_once, attr_rc) != hipSuccess) return attr_rc;
    const int num_tiles = Lay.NT;
    const int groups = (num_tiles + 3) / 4;
    const dim3 grid(groups < 256 ? groups : 256);      // one workgroup per compute unit
    launch(prof, k_lmhead_skinny<KH, MT, FUSE>, grid, dim3(kSkinnyThreads), lds, s, M, c.V, c.n, Lay.NT, num_tiles,
           static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(H), temperature, logits, pm, ps, tail);
    return hipSuccess;
}

// Dispatch over (k-blocks per wave, row blocks, fused sampler or not); chunked = the K-chunked kernel.
static hipError_t launch_skinny_any(bool chunked, int KH, const ProfScope* prof, const tabed_cfg& c, const WsLayout& Lay,
                                    int M, const void* W, const void* H, const float* temperature, float* logits,
                                    float* pm, float* ps, const TailArgs& tail, hipStream_t s) {
    const int MT = (M + 31) / 32;
    const bool fuse = tail.ticket != nullptr;
#define TABED_SKINNY_CASE(FN_, KH_)                                                                               \
    if (KH == KH_) {                                                                                              \
        if (MT == 1) return fuse ? FN_<KH_, 1, true>(prof, c, Lay, M, W, H, temperature, logits, pm, ps, tail, s) \
                                 : FN_<KH_, 1, false>(prof, c, Lay, M, W, H, temperature, logits, pm, ps, tail, s); \
        return fuse ? FN_<KH_, 2, true>(prof, c, Lay, M, W, H, temperature, logits, pm, ps, tail, s)              \
                    : FN_<KH_, 2, false>(prof, c, Lay, M, W, H, temperature, logits, pm, ps, tail, s);            \
    }
    if (chunked) {
        TABED_SKINNY_CASE(launch_skinny_kc_t, 4) TABED_SKINNY_CASE(launch_skinny_kc_t, 6) TABED_SKINNY_CASE(launch_skinny_kc_t, 7)
    } else {
        TABED_SKINNY_CASE(launch_skinny_t, 4) TABED_SKINNY_CASE(launch_skinny_t, 6) TABED_SKINNY_CASE(launch_skinny_t, 7)
        TABED_SKINNY_CASE(launch_skinny_t, 8)
    }
#undef TABED_SKINNY_CASE
    return hipErrorInvalidValue;
}

static bool skinny_applies(const tabed_cfg& c, int M) {
    if (c.w_dtype != 1 || M > 64 || c.d % 128 != 0) return false;
    const int KH = c.d / 128, MT = (M + 31) / 32;
    if (KH != 4 && KH != 6 && KH != 7 && KH != 8) return false;
    return skinny_lds_bytes(KH, MT) <= 160 * 1024;
}

hipError_t launch_lmhead(const tabed_cfg& c, const WsLayout& Lay, char* ws, const void* W, const void* H,
                         const float* temperature, float* logits, const SamplerIo* io, bool* fused, hipStream_t s) {
    ProfScope prof(TABED_K_LMHEAD, s);
    float* pm = reinterpret_cast<float*>(ws + Lay.off_pm);
    float* ps = reinterpret_cast<float*>(ws + Lay.off_ps);
    const int M = Lay.M;
    if (fused != nullptr) *fused = false;
    const bool plain_skinny = skinny_applies(c, M);
    const int kc = plain_skinny ? 0 : skinny_kc_kh(c, M);
    if (c.w_dtype == 0) {
        const dim3 grid(Lay.NT, (M + 7) / 8);
        launch(&prof, k_lmhead_f32, grid, dim3(kBlock), 0, s, M, c.d, c.V, c.n, Lay.NT,
                           static_cast<const float*>(W), static_cast<const float*>(H), temperature, logits, pm, ps);
    } else if (plain_skinny || kc != 0) {
        const int KH = plain_skinny ? c.d / 128 : kc, MT = (M + 31) / 32;
        TailArgs tail{};
        if (io != nullptr && fused != nullptr && tail_fits(c, Lay, KH, MT)) {
            tail.B = c.B; tail.gamma = c.gamma; tail.pos = io->pos; tail.NG = Lay.NG;
            tail.greedy_here = c.sampling_only ? 1 : 0;
            tail.seed = c.seed; tail.round = io->round;
            tail.weights = io->weights; tail.u_draft = io->u_draft;
            tail.draft_lse = io->draft_lse; tail.draft_tokens = io->draft_tokens; tail.draft_q = io->draft_q;
            tail.flags = io->flags;
            tail.gsum = reinterpret_cast<unsigned long long*>(ws + Lay.off_gsum);
            tail.ticket = reinterpret_cast<uint32_t*>(ws + Lay.off_tickets) + 1 * c.B;
            *fused = true;
        }
        const hipError_t e = launch_skinny_any(!plain_skinny, KH, &prof, c, Lay, M, W, H, temperature, logits, pm, ps, tail, s);
        if (e != hipSuccess) return e;
    } else if (M > 64 && c.d % 64 == 0) {
        static std::once_flag attr_once;                   // raise the dynamic-LDS limit once
        static hipError_t attr_rc = hipSuccess;
        const size_t lds = 2 * (size_t)kLargeStage;
        if (raise_lds_limit(&k_lmhead_large<kLargeWaves>, lds, attr_once, attr_rc) != hipSuccess) return attr_rc;
        const int mblocks = (M + kLBM - 1) / kLBM, nblocks = (c.V + kLBN - 1) / kLBN;
        const int nrounds = (nblocks + 7) / 8;             // vocabulary blocks are dealt to the 8 XCDs in rounds
        const dim3 grid(nrounds * mblocks * 8);
        launch(&prof, k_lmhead_large<kLargeWaves>, grid, dim3(kLargeWaves * 64), lds, s, M, c.d, c.V, c.n, Lay.NT, mblocks,
               static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(H), temperature, logits, pm, ps);
    } else {
        const dim3 grid((c.V + kBN - 1) / kBN, (M + kBM - 1) / kBM);
        launch(&prof, k_lmhead_bf16, grid, dim3(kBlock), 0, s, M, c.d, c.V, c.n, Lay.NT,
                           static_cast<const __hip_bfloat16*>(W), static_cast<const __hip_bfloat16*>(H),
                           temperature, logits, pm, ps);
    }
    return hipGetLastError();
}

}  // namespace tabed
