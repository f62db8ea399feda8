// LM head of the n batched drafts (Alg. 1 (draft forward), last layer of the shared draft model):
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
            if (m_base + mr < M)
                __builtin_nontemporal_store(f32x4{val.x, val.y, val.z, val.w},
                                            reinterpret_cast<f32x4*>(L + (size_t)(m_base + mr) * V + v_base + 4 * q));
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
            if (v < V) row[v] = acc[4 * g + e];
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

template <int KH, int MT>
__global__ __launch_bounds__(kSkinnyThreads) void k_lmhead_skinny(int M, int V, int n, int NT, int num_tiles,
                                                                  const uint16_t* __restrict__ W,
                                                                  const uint16_t* __restrict__ H,
                                                                  const float* __restrict__ temperature,
                                                                  float* __restrict__ L, float* __restrict__ pm,
                                                                  float* __restrict__ ps) {
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
            store_tile_32x32_t(fin, (MT == 2) ? khalf * 32 : 0, this_tile * 32, M, V, NT, s_invt, L, pm, ps, patch, s_pstage, pair);
        // the four tiles of this group sit side by side in a row of the partial tables: 16 bytes per row
        lds_barrier();
        if (tid < 128 && (tid & 63) < M) {
            const int arr = tid >> 6, row = tid & 63, t0 = g * 4;
            float* dst = (arr == 0 ? pm : ps) + (size_t)row * NT + t0;
            const float* srcp = s_pstage + (arr * 64 + row) * 4;
            if ((NT & 3) == 0 && t0 + 3 < NT) *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(srcp);
            else for (int q = 0; q < 4; ++q) if (t0 + q < NT) dst[q] = srcp[q];
        }
        if (!more) break;
#pragma unroll
        for (int i = 0; i < 4; ++i) src[i] = nsrc[i];
    }
}

// ---------------------------------------------------------------- bf16, skinny M, larger hidden sizes
// Same design as k_lmhead_skinny for hidden sizes whose H (64 x d) does not fit LDS: K is walked in chunks of
// KH*128, and LDS holds one chunk of H at a time.  The next chunk of H is requested into registers at the
// start of a chunk's k-loop and written to LDS between two LDS-only barriers at its end; the W request
// stream (kPF k-blocks ahead) runs straight across chunk boundaries.  d = nchunks * KH * 128.
template <int KH, int MT>
__global__ __launch_bounds__(kSkinnyThreads) void k_lmhead_skinny_kc(int M, int V, int n, int NT, int num_tiles,
                                                                     int nchunks,
                                                                     const uint16_t* __restrict__ W,
                                                                     const uint16_t* __restrict__ H,
                                                                     const float* __restrict__ temperature,
                                                                     float* __restrict__ L, float* __restrict__ pm,
                                                                     float* __restrict__ ps) {
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
            store_tile_32x32_t(fin, (MT == 2) ? khalf * 32 : 0, this_tile * 32, M, V, NT, s_invt, L, pm, ps, patch, s_pstage, pair);
        // the four tiles of this group sit side by side in a row of the partial tables: 16 bytes per row
        lds_barrier();
        if (tid < 128 && (tid & 63) < M) {
            const int arr = tid >> 6, row = tid & 63, t0 = g * 4;
            float* dst = (arr == 0 ? pm : ps) + (size_t)row * NT + t0;
            const float* srcp = s_pstage + (arr * 64 + row) * 4;
            if ((NT & 3) == 0 && t0 + 3 < NT) *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(srcp);
            else for (int q = 0; q < 4; ++q) if (t0 + q < NT) dst[q] = srcp[q];
        }
        if (!more) break;
#pragma unroll
        for (int i = 0; i < 4; ++i) src[i] = nsrc[i];
    }
}

// ---------------------------------------------------------------- bf16, many rows (M > 64): MFMA-bound tiled GEMM
// With hundreds of rows (stress shape: n*B = 512) the LM head is a real GEMM: 2*M*d*V flops against one
// pass over W.  Workgroup tile 256 (rows) x 256 (vocabulary) x 64 (k), 8 waves, each wave a 128 (rows) x 64
// (vocabulary) block (2 x 4 MFMA 32x32x16 tiles, W as the row operand so the accumulator is
// [vocabulary][row] and the cheap transposed epilogue applies).  Both operands are staged through LDS in two
// buffers; the operand fragments of k-step s+1 are read from LDS while the MFMAs of k-step s run, and the
// global loads of k-block i+1 are in flight (one register set) while k-block i-1 and i are multiplied --
// one barrier per k-block.  A k-block of 64 is one whole 128-byte line of every row (measured 4.5 % faster than
// k-blocks of 32 with two register sets: 318 against 334 us at the stress shape).  Rows padded by 16 bytes
// against bank conflicts.  Workgroups are numbered so that
// the row blocks that share a vocabulary block run back to back on the same XCD (workgroup w goes to XCD
// w % 8): W is then read from HBM once and from L2 afterwards.
constexpr int kLBM = 256, kLBN = 256, kLBK = 64, kLRow = (kLBK + 8) * 2;   // LDS row stride in bytes (144)
constexpr int kLCh = kLBK / 8;                                              // 16-byte chunks per row of a k-block
constexpr int kLargeStage = (kLBM + kLBN) * kLRow;                          // bytes per buffer (73728)

// Eight waves per workgroup, each 128 rows x 64 vocabulary entries, two waves per SIMD.  (Four waves of 128 x 128 with
// register staging spill ~300 registers; four waves fed by global_load_lds measured no faster: the loop is bound by
// how fast a workgroup pulls its operand tiles, 1 byte per 128 flop at this tile size, through L1 from L2.)
constexpr int kLargeWaves = 8;

__global__ __launch_bounds__(kLargeWaves * 64) void k_lmhead_large(int M, int d, int V, int n, int NT, int mblocks,
                                                                const uint16_t* __restrict__ W,
                                                                const uint16_t* __restrict__ H,
                                                                const float* __restrict__ temperature,
                                                                float* __restrict__ L, float* __restrict__ pm,
                                                                float* __restrict__ ps) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ float s_invt[kLBM];
    constexpr int NW = kLargeWaves;
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

    // ---- global -> register staging: kLWPieces of W and kLHPieces of H per thread (16 bytes each), one k-block
    //      ahead of the one in LDS.
    u32x4 rw[kLWPieces], rh[kLHPieces];
    auto fetch = [&](int kb) {
        const int k = kb * kLBK;
#pragma unroll
        for (int t = 0; t < kLWPieces; ++t) {
            const int q = tid + t * kLargeThreads, row = q / kLCh, c = q % kLCh;
            const int v = min(v0 + row, V - 1);           // clamped rows are masked in the epilogue
            rw[t] = *reinterpret_cast<const u32x4*>(W + (size_t)v * d + k + c * 8);
        }
#pragma unroll
        for (int t = 0; t < kLHPieces; ++t) {
            const int q = tid + t * kLargeThreads, row = q / kLCh, c = q % kLCh;
            const int m = min(m0 + row, M - 1);
            rh[t] = *reinterpret_cast<const u32x4*>(H + (size_t)m * d + k + c * 8);
        }
    };
    auto stash = [&](int buf) {
        unsigned char* sW = lds + buf * kLargeStage;
        unsigned char* sH = sW + kLBN * kLRow;
#pragma unroll
        for (int t = 0; t < kLWPieces; ++t) {
            const int q = tid + t * kLargeThreads, row = q / kLCh, c = q % kLCh;
            *reinterpret_cast<u32x4*>(sW + row * kLRow + c * 16) = rw[t];
        }
#pragma unroll
        for (int t = 0; t < kLHPieces; ++t) {
            const int q = tid + t * kLargeThreads, row = q / kLCh, c = q % kLCh;
            *reinterpret_cast<u32x4*>(sH + row * kLRow + c * 16) = rh[t];
        }
    };

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

    // k-block kb+1 is requested while k-block kb-1 is multiplied and written to LDS after k-block kb: its loads have
    // one multiply (about 2000 MFMA cycles per SIMD, more than an L2 round trip) to arrive.
    const int KB = d / kLBK;
    fetch(0);
    stash(0);
    if (1 < KB) fetch(1);
    lds_barrier();
    for (int kb = 0; kb < KB; ++kb) {
        multiply(kb & 1);
        if (kb + 1 < KB) stash((kb + 1) & 1);
        if (kb + 2 < KB) fetch(kb + 2);
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

template <int KH, int MT>
static hipError_t launch_skinny_kc_t(const ProfScope* prof, const tabed_cfg& c, const WsLayout& Lay, int M, const void* W,
                               const void* H, const float* temperature, float* logits, float* pm, float* ps,
                               hipStream_t s) {
    const size_t lds = (size_t)MT * 32 * (KH * 256 + 16) + (size_t)kSkinnyWaves * kPatchBytes;
    static std::once_flag attr_once;
    static hipError_t attr_rc = hipSuccess;
    if (raise_lds_limit(&k_lmhead_skinny_kc<KH, MT>, lds, attr_once, attr_rc) != hipSuccess) return attr_rc;
    const int num_tiles = Lay.NT, groups = (num_tiles + 3) / 4;
    const dim3 grid(groups < 256 ? groups : 256);
    launch(prof, k_lmhead_skinny_kc<KH, MT>, grid, dim3(kSkinnyThreads), lds, s, M, c.V, c.n, Lay.NT, num_tiles,
           c.d / (KH * 128), static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(H), temperature, logits, pm, ps);
    return hipSuccess;
}

static hipError_t launch_skinny_kc(const ProfScope* prof, int KH, const tabed_cfg& c, const WsLayout& Lay, int M,
                             const void* W, const void* H, const float* temperature, float* logits, float* pm,
                             float* ps, hipStream_t s) {
    const int MT = (M + 31) / 32;
#define TABED_SKINNY_KC(KH_)                                                                              \
    if (KH == KH_) {                                                                                      \
        if (MT == 1) return launch_skinny_kc_t<KH_, 1>(prof, c, Lay, M, W, H, temperature, logits, pm, ps, s);   \
        else         return launch_skinny_kc_t<KH_, 2>(prof, c, Lay, M, W, H, temperature, logits, pm, ps, s);   \
    }
    TABED_SKINNY_KC(4) TABED_SKINNY_KC(6) TABED_SKINNY_KC(7)
#undef TABED_SKINNY_KC
    return hipErrorInvalidValue;
}

static bool skinny_applies(const tabed_cfg& c, int M) {
    if (c.w_dtype != 1 || M > 64 || c.d % 128 != 0) return false;
    const int KH = c.d / 128, MT = (M + 31) / 32;
    if (KH != 4 && KH != 6 && KH != 7 && KH != 8) return false;
    const size_t lds = (size_t)MT * 32 * (c.d * 2 + 16) + (size_t)kSkinnyWaves * kPatchBytes;
    return lds <= 160 * 1024;
}

template <int KH, int MT>
static hipError_t launch_skinny_t(const ProfScope* prof, const tabed_cfg& c, const WsLayout& Lay, int M, const void* W, const void* H,
                            const float* temperature, float* logits, float* pm, float* ps, hipStream_t s) {
    const size_t lds = (size_t)MT * 32 * (KH * 256 + 16) + (size_t)kSkinnyWaves * kPatchBytes;
    static std::once_flag attr_once;                   // raise the dynamic-LDS limit of this instantiation once
    static hipError_t attr_rc = hipSuccess;
    if (raise_lds_limit(&k_lmhead_skinny<KH, MT>, lds, attr_once, attr_rc) != hipSuccess) return attr_rc;
    const int num_tiles = Lay.NT;
    int cus = 256;
    const int groups = (num_tiles + 3) / 4;
    const dim3 grid(groups < cus ? groups : cus);
    launch(prof, k_lmhead_skinny<KH, MT>, grid, dim3(kSkinnyThreads), lds, s, M, c.V, c.n, Lay.NT, num_tiles,
                       static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(H), temperature, logits, pm, ps);
    return hipSuccess;
}

static hipError_t launch_skinny(const ProfScope* prof, const tabed_cfg& c, const WsLayout& Lay, int M, const void* W, const void* H,
                          const float* temperature, float* logits, float* pm, float* ps, hipStream_t s) {
    const int KH = c.d / 128, MT = (M + 31) / 32;
#define TABED_SKINNY(KH_)                                                                              \
    if (KH == KH_) {                                                                                   \
        if (MT == 1) return launch_skinny_t<KH_, 1>(prof, c, Lay, M, W, H, temperature, logits, pm, ps, s);  \
        else         return launch_skinny_t<KH_, 2>(prof, c, Lay, M, W, H, temperature, logits, pm, ps, s);  \
    }
    TABED_SKINNY(4) TABED_SKINNY(6) TABED_SKINNY(7) TABED_SKINNY(8)
#undef TABED_SKINNY
    return hipErrorInvalidValue;
}

hipError_t launch_lmhead(const tabed_cfg& c, const WsLayout& Lay, char* ws, const void* W, const void* H,
                         const float* temperature, float* logits, hipStream_t s, int prof_id) {
    ProfScope prof(prof_id, s);
    float* pm = reinterpret_cast<float*>(ws + Lay.off_pm);
    float* ps = reinterpret_cast<float*>(ws + Lay.off_ps);
    const int M = Lay.M;
    if (c.w_dtype == 0) {
        const dim3 grid(Lay.NT, (M + 7) / 8);
        launch(&prof, k_lmhead_f32, grid, dim3(kBlock), 0, s, M, c.d, c.V, c.n, Lay.NT,
                           static_cast<const float*>(W), static_cast<const float*>(H), temperature, logits, pm, ps);
    } else if (skinny_applies(c, M)) {
        const hipError_t e = launch_skinny(&prof, c, Lay, M, W, H, temperature, logits, pm, ps, s);
        if (e != hipSuccess) return e;
    } else if (skinny_kc_kh(c, M) != 0) {
        const hipError_t e = launch_skinny_kc(&prof, skinny_kc_kh(c, M), c, Lay, M, W, H, temperature, logits, pm, ps, s);
        if (e != hipSuccess) return e;
    } else if (M > 64 && c.d % 64 == 0) {
        static std::once_flag attr_once;                   // raise the dynamic-LDS limit once
        static hipError_t attr_rc = hipSuccess;
        const size_t lds = 2 * (size_t)kLargeStage;
        if (raise_lds_limit(&k_lmhead_large, lds, attr_once, attr_rc) != hipSuccess) return attr_rc;
        const int mblocks = (M + kLBM - 1) / kLBM, nblocks = (c.V + kLBN - 1) / kLBN;
        const int nrounds = (nblocks + 7) / 8;             // vocabulary blocks are dealt to the 8 XCDs in rounds
        const dim3 grid(nrounds * mblocks * 8);
        launch(&prof, k_lmhead_large, grid, dim3(kLargeWaves * 64), lds, s, M, c.d, c.V, c.n, Lay.NT, mblocks,
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
