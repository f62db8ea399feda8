// LM head of the n batched drafts (Alg. 1 line 5, last layer of the shared draft model):
//   L[r, v] = sum_k H[r, k] * W[v, k],   r = b*n + j  (M = n*B rows),
// with the first half of the per-draft softmax fused into the epilogue: for every row and every 32-wide
// vocabulary tile the kernel also writes  pm = max_v s(v)  and  ps = sum_v exp(s(v) - pm),  s = L / T_b.
// gfx950: bf16 operands go through v_mfma_f32_32x32x16_bf16 (fp32 accumulate); fp32 operands (the tiny
// correctness configuration) use plain FMAs.
#include <hip/hip_bf16.h>

#include "device_utils.h"
#include "internal.h"

namespace tabed {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

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
// 8*(r/4) + 4*(lane/32) + r%4.  Writes logits and the tile's softmax partials.
__device__ __forceinline__ void store_tile_32x32(const f32x16& acc, int m_base, int v_base, int M, int V, int n,
                                                 int NT, const float* __restrict__ temperature,
                                                 float* __restrict__ L, float* __restrict__ pm,
                                                 float* __restrict__ ps) {
    if (v_base >= V) return;
    const int lane = threadIdx.x & 63;
    const int col = lane & 31, half = lane >> 5;
    const int v = v_base + col;
    const int tile = v_base / kTileV;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = m_base + 8 * (r / 4) + 4 * half + (r % 4);
        const bool live = (m < M);          // uniform over the half-wave
        const float x = acc[r];
        float s = -INFINITY;
        if (live && v < V) {
            L[(size_t)m * V + v] = x;
            s = x * row_inv_temperature(temperature, m, n);
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
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int v0 = blockIdx.x * kBN, m0 = blockIdx.y * kBM;
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
    store_tile_32x32(acc, m0 + wm * 32, v0 + wn * 32, M, V, n, NT, temperature, L, pm, ps);
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

hipError_t launch_lmhead(const tabed_cfg& c, const WsLayout& Lay, char* ws, const void* W, const void* H,
                         const float* temperature, float* logits, hipStream_t s) {
    ProfScope prof(TABED_K_LMHEAD, s);
    float* pm = reinterpret_cast<float*>(ws + Lay.off_pm);
    float* ps = reinterpret_cast<float*>(ws + Lay.off_ps);
    const int M = Lay.M;
    if (c.w_dtype == 0) {
        const dim3 grid(Lay.NT, (M + 7) / 8);
        hipLaunchKernelGGL(k_lmhead_f32, grid, dim3(kBlock), 0, s, M, c.d, c.V, c.n, Lay.NT,
                           static_cast<const float*>(W), static_cast<const float*>(H), temperature, logits, pm, ps);
    } else {
        const dim3 grid((c.V + kBN - 1) / kBN, (M + kBM - 1) / kBM);
        hipLaunchKernelGGL(k_lmhead_bf16, grid, dim3(kBlock), 0, s, M, c.d, c.V, c.n, Lay.NT,
                           static_cast<const __hip_bfloat16*>(W), static_cast<const __hip_bfloat16*>(H),
                           temperature, logits, pm, ps);
    }
    return hipGetLastError();
}

}  // namespace tabed
