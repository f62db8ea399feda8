// Draft-model body in front of the LM head (Sec. 5.1 "Ensemble learning via Batched Inference", Sec. 4.1 "Target and
// Draft Models"): one decode step of a LLaMA-style decoder for the n*B rows of the batch of drafting methods, each
// with its own key / value cache.  At 64 rows every projection streams a few megabytes of weights and is bound by
// launch and latency, not bandwidth: the contraction is split into ranges so that a few hundred workgroups have
// their loads in flight at once, the partial sums go to slabs that the consumer of the projection (rotary
// embedding + cache append + attention, residual + RMSNorm, SwiGLU) adds in a fixed order.  Storage points: bf16 for
// weights, caches and everything that feeds a projection; fp32 for the residual stream and the projections'
// results.  Shapes the split kernels do not take go through the LM head's kernels (any [rows,K] x [N,K]^T -> fp32).
#include <hip/hip_bf16.h>

#include "device_utils.h"
#include "internal.h"

namespace tabed {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4b;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {            // round to nearest even
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (uint16_t)((u + (((u >> 16) & 1u) + 0x7FFFu)) >> 16);
}

__device__ __forceinline__ float block_sum_f32(float v, float* lds4) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
    __syncthreads();
    const float r = (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
    __syncthreads();
    return r;
}

// A projection's result arrives as `ks` partial sums over disjoint ranges of the contraction index (slabs, `slab`
// floats apart), summed here in slab order: the split keeps every compute unit busy on matrices this small, and
// a fixed order keeps the result reproducible bit for bit.
__device__ __forceinline__ float slab_sum(const float* __restrict__ p, int ks, size_t slab) {
    float v = p[0];
    for (int j = 1; j < ks; ++j) v += p[(size_t)j * slab];
    return v;
}

// ---------------------------------------------------------------- embedding + first RMSNorm
__global__ __launch_bounds__(kBlock) void k_body_embed_norm(int d, int V, float eps, const int32_t* __restrict__ token_src,
                                                            int token_stride, int rows_per_token,
                                                            const uint16_t* __restrict__ embed, const float* __restrict__ g,
                                                            float* __restrict__ x, uint16_t* __restrict__ hb) {
    __shared__ float s_red[kWavesPerBlock];
    const int r = blockIdx.x;
    int tok = token_src[(size_t)(r / rows_per_token) * token_stride];
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
    const uint16_t* e = embed + (size_t)tok * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += kBlock) {
        const float v = bf16_bits_to_f32(e[i]);
        x[(size_t)r * d + i] = v;
        ss += v * v;
    }
    const float inv = 1.f / sqrtf(block_sum_f32(ss, s_red) / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += kBlock)
        hb[(size_t)r * d + i] = f32_to_bf16_bits(bf16_bits_to_f32(e[i]) * inv * g[i]);
}

// ---------------------------------------------------------------- residual + RMSNorm (+ position advance at the end of a step)
// One workgroup per row, a thread per four consecutive elements; the slabs are requested eight at a time so that
// a row costs two or three trips to memory, not one per slab.
constexpr int kSlabBatch = 8;
__global__ __launch_bounds__(kBlock) void k_body_add_norm(int d, float eps, int ks, size_t slab, float* __restrict__ x,
                                                          const float* __restrict__ y /* [ks][rows,d] */,
                                                          const float* __restrict__ g, uint16_t* __restrict__ out,
                                                          int32_t* ctx_len_advance) {
    __shared__ float s_red[kWavesPerBlock];
    extern __shared__ __attribute__((aligned(16))) float4 s_row[];        // [d / 4] the row after the addition
    const int r = blockIdx.x;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d / 4; i += kBlock) {
        float4 v = *reinterpret_cast<const float4*>(x + (size_t)r * d + 4 * i);
        const float* yp = y + (size_t)r * d + 4 * i;
        for (int j0 = 0; j0 < ks; j0 += kSlabBatch) {
            float4 part[kSlabBatch];
#pragma unroll
            for (int u = 0; u < kSlabBatch; ++u)                             // past the last slab: re-read it, add nothing
                part[u] = *reinterpret_cast<const float4*>(yp + (size_t)min(j0 + u, ks - 1) * slab);
#pragma unroll
            for (int u = 0; u < kSlabBatch; ++u)
                if (j0 + u < ks) { v.x += part[u].x; v.y += part[u].y; v.z += part[u].z; v.w += part[u].w; }
        }
        *reinterpret_cast<float4*>(x + (size_t)r * d + 4 * i) = v;
        s_row[i] = v;
        ss += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
    }
    const float inv = 1.f / sqrtf(block_sum_f32(ss, s_red) / (float)d + eps);
    for (int i = threadIdx.x; i < d / 4; i += kBlock) {
        const float4 v = s_row[i], gg = *reinterpret_cast<const float4*>(g + 4 * i);
        const uint32_t lo = f32_to_bf16_bits(v.x * inv * gg.x) | ((uint32_t)f32_to_bf16_bits(v.y * inv * gg.y) << 16);
        const uint32_t hi = f32_to_bf16_bits(v.z * inv * gg.z) | ((uint32_t)f32_to_bf16_bits(v.w * inv * gg.w) << 16);
        *reinterpret_cast<uint2*>(out + (size_t)r * d + 4 * i) = make_uint2(lo, hi);
    }
    if (ctx_len_advance != nullptr && threadIdx.x == 0) ctx_len_advance[r] += 1;
}

// ---------------------------------------------------------------- SwiGLU: silu(gate) * up
__global__ __launch_bounds__(kBlock) void k_body_silu_mul(int rows, int d_ff, int ks, size_t slab,
                                                          const float* __restrict__ gu /* [ks][rows, 2 d_ff] */,
                                                          uint16_t* __restrict__ act) {
    const size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= (size_t)rows * d_ff) return;
    const size_t r = i / d_ff, f = i % d_ff;
    const float gte = slab_sum(gu + r * 2 * d_ff + f, ks, slab), up = slab_sum(gu + r * 2 * d_ff + d_ff + f, ks, slab);
    act[i] = f32_to_bf16_bits(gte / (1.f + __expf(-gte)) * up);
}

// ---------------------------------------------------------------- projection for <= 64 rows, split over the contraction
// Y[ks][m][n] = sum over the ks-th K range of X[m][k] W[n][k].  One workgroup = one 32-column tile of the result
// and one K range; its four waves take a quarter of the range each, reading W and X straight into the MFMA operand
// layout (lane = row, 8 consecutive k: 32 bytes per row and instruction, whole lines over four instructions),
// and meet through LDS: wave w sums, in wave order, the quarter of the accumulator it then stores.  The matrices
// are a few megabytes: what matters is that a few hundred workgroups each have their loads in flight at once.
constexpr int kProjGroup = 4;                         // k-steps (of 16) requested together
template <int MT>
__global__ __launch_bounds__(kBlock) void k_body_proj(int M, int N, int K, int steps_per_wave,
                                                      const uint16_t* __restrict__ X, const uint16_t* __restrict__ W,
                                                      float* __restrict__ Y, size_t slab) {
    __shared__ __attribute__((aligned(16))) float4 s_acc[kWavesPerBlock][MT][4][kWave];
    const int tile = blockIdx.x, ks = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nn = lane & 31, half = lane >> 5;
    const int k0 = ((ks * kWavesPerBlock + wave) * steps_per_wave) * 16 + half * 8;
    const uint16_t* wp = W + (size_t)min(tile * 32 + nn, N - 1) * K + k0;
    const uint16_t* xp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xp[mt] = X + (size_t)min(mt * 32 + nn, M - 1) * K + k0;
    f32x16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
    for (int s0 = 0; s0 < steps_per_wave; s0 += kProjGroup) {
        bf16x8 wv[kProjGroup], xv[kProjGroup][MT];
#pragma unroll
        for (int q = 0; q < kProjGroup; ++q) {
            const int s = min(s0 + q, steps_per_wave - 1);          // a short last group re-reads its last step
            wv[q] = *reinterpret_cast<const bf16x8*>(wp + s * 16);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xv[q][mt] = *reinterpret_cast<const bf16x8*>(xp[mt] + s * 16);
        }
#pragma unroll
        for (int q = 0; q < kProjGroup; ++q) {
            if (s0 + q < steps_per_wave) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv[q], xv[q][mt], acc[mt], 0, 0, 0);
            }
        }
    }
    // accumulator: lane holds result row m = nn (+ 32 mt), columns n = 8 g + 4 half + 0..3 in registers 4 g .. 4 g + 3
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int g = 0; g < 4; ++g)
            s_acc[wave][mt][g][lane] = make_float4(acc[mt][4 * g], acc[mt][4 * g + 1], acc[mt][4 * g + 2], acc[mt][4 * g + 3]);
    __syncthreads();
    const int g = wave;                                              // this wave finishes column group g
    const int n = tile * 32 + 8 * g + 4 * half;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        float4 t = s_acc[0][mt][g][lane];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) {
            const float4 o = s_acc[w][mt][g][lane];
            t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w;
        }
        const int m = mt * 32 + nn;
        if (m < M && n < N) *reinterpret_cast<float4*>(Y + (size_t)ks * slab + (size_t)m * N + n) = t;   // N % 4 == 0
    }
}

// ---------------------------------------------------------------- projection for <= 64 rows, wide results
// The same contraction for results wide enough to fill the chip with fewer K ranges: one workgroup = four
// 32-column tiles (one per wave) and one K range of KG * 64.  The X chunk of the range is staged once into LDS
// and shared by the four waves (all workgroups read the same few X lines, so fetching them once per workgroup
// instead of once per wave matters); every wave requests all of its W before anything else.
template <int MT, int KG>
__global__ __launch_bounds__(kBlock) void k_body_proj_wide(int M, int N, int K, const uint16_t* __restrict__ X,
                                                           const uint16_t* __restrict__ W, float* __restrict__ Y, size_t slab) {
    constexpr int KC = KG * 64, CH = KC / 8, XROW = KC * 2 + 16;          // chunk width, its 16-byte pieces, padded LDS row
    __shared__ __attribute__((aligned(16))) unsigned char s_x[MT * 32 * XROW];
    const int ks = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nn = lane & 31, half = lane >> 5;
    const int tile = blockIdx.x * kWavesPerBlock + wave;
    const int kbase = ks * KC;
    const uint16_t* wp = W + (size_t)min(tile * 32 + nn, N - 1) * K + kbase + half * 8;
    bf16x8 wv[KG * 4];
#pragma unroll
    for (int q = 0; q < KG * 4; ++q) wv[q] = *reinterpret_cast<const bf16x8*>(wp + q * 16);
    constexpr int kPieces = MT * 32 * CH, kPer = (kPieces + kBlock - 1) / kBlock;
    u32x4b xr[kPer];
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int p = min(tid + q * kBlock, kPieces - 1), row = min(p / CH, M - 1), c = p % CH;
        xr[q] = *reinterpret_cast<const u32x4b*>(X + (size_t)row * K + kbase + c * 8);
    }
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int p = tid + q * kBlock;
        if (p < kPieces) *reinterpret_cast<u32x4b*>(s_x + (p / CH) * XROW + (p % CH) * 16) = xr[q];
    }
    __syncthreads();
    f32x16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
#pragma unroll
    for (int q = 0; q < KG * 4; ++q)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const bf16x8 xv = *reinterpret_cast<const bf16x8*>(s_x + (mt * 32 + nn) * XROW + (2 * q + half) * 16);
            acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv[q], xv, acc[mt], 0, 0, 0);
        }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 32 + nn;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n = tile * 32 + 8 * g + 4 * half;
            if (m < M && n < N)
                *reinterpret_cast<float4*>(Y + (size_t)ks * slab + (size_t)m * N + n) =
                    make_float4(acc[mt][4 * g], acc[mt][4 * g + 1], acc[mt][4 * g + 2], acc[mt][4 * g + 3]);
        }
    }
}

// ---------------------------------------------------------------- rotary embedding + cache append + attention
// Grid (head, row), four waves.  The rotation is done in fp64 (a position times a tiny frequency loses digits in
// fp32).  A key's (value's) head slice is hd contiguous bf16: LPK = hd / 8 lanes read it as 16-byte pieces, so one
// wave instruction fetches 64 / LPK whole slices, and every lane keeps four such loads in flight.  Scores: dot
// product over the LPK lanes, softmax over the workgroup through LDS.  Values: every lane accumulates its 8
// dimensions over the keys it sees; lanes, then waves, are summed in a fixed order.
constexpr int kAttnUnroll = 4;
template <int LPK>
__global__ __launch_bounds__(kBlock) void k_body_rope_attn(int d, int max_ctx, double theta, int ks, size_t slab,
                                                           const float* __restrict__ qkv /* [ks][rows,3d] */,
                                                           const int32_t* __restrict__ ctx_len,
                                                           uint16_t* __restrict__ kc /* [rows,max_ctx,d] of this layer */,
                                                           uint16_t* __restrict__ vc, uint16_t* __restrict__ att /* [rows,d] */) {
    constexpr int hd = LPK * 8, G = kWave / LPK;                          // G keys per wave instruction
    extern __shared__ __attribute__((aligned(16))) float s_sc[];          // [max_ctx] scores, then probabilities
    __shared__ float s_q[hd], s_part[kWavesPerBlock][hd];
    __shared__ float s_redf[kWavesPerBlock];
    const int hh = blockIdx.x, r = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int pos = ctx_len[r];
    pos = pos < 0 ? 0 : (pos >= max_ctx ? max_ctx - 1 : pos);            // never write outside the row's cache
    const float* q = qkv + (size_t)r * 3 * d + hh * hd;
    const float* k = q + d;
    const float* v = q + 2 * d;
    uint16_t* Kr = kc + (size_t)r * max_ctx * d + hh * hd;                // key t of this head: Kr + t * d
    uint16_t* Vr = vc + (size_t)r * max_ctx * d + hh * hd;
    if (tid < hd / 2) {
        const int i = tid;
        const double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
        double sn, cs;
        sincos(ang, &sn, &cs);
        const double q0 = (double)slab_sum(q + i, ks, slab), q1 = (double)slab_sum(q + i + hd / 2, ks, slab);
        const double k0 = (double)slab_sum(k + i, ks, slab), k1 = (double)slab_sum(k + i + hd / 2, ks, slab);
        s_q[i] = (float)(q0 * cs - q1 * sn);
        s_q[i + hd / 2] = (float)(q1 * cs + q0 * sn);
        Kr[(size_t)pos * d + i] = f32_to_bf16_bits((float)(k0 * cs - k1 * sn));
        Kr[(size_t)pos * d + i + hd / 2] = f32_to_bf16_bits((float)(k1 * cs + k0 * sn));
    }
    if (tid >= 128 && tid < 128 + hd) {
        const int i = tid - 128;
        Vr[(size_t)pos * d + i] = f32_to_bf16_bits(slab_sum(v + i, ks, slab));
    }
    __syncthreads();                    // the new key and value are read back below by other waves of this workgroup
    const int g = lane / LPK, c = lane % LPK;
    float qr[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) qr[e] = s_q[c * 8 + e];
    const float scale = 1.f / sqrtf((float)hd);
    constexpr int kStride = kWavesPerBlock * G;                           // keys per workgroup instruction
    float mx = -INFINITY;
    for (int base = wave * G + g; base - g - wave * G <= pos; base += kStride * kAttnUnroll) {
        u32x4b w4[kAttnUnroll];
#pragma unroll
        for (int u = 0; u < kAttnUnroll; ++u)                            // keys past the end re-read key pos
            w4[u] = *reinterpret_cast<const u32x4b*>(Kr + (size_t)min(base + u * kStride, pos) * d + c * 8);
#pragma unroll
        for (int u = 0; u < kAttnUnroll; ++u) {
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc += qr[2 * e] * __builtin_bit_cast(float, w4[u][e] << 16);
                acc += qr[2 * e + 1] * __builtin_bit_cast(float, w4[u][e] & 0xffff0000u);
            }
#pragma unroll
            for (int off = 1; off < LPK; off <<= 1) acc += __shfl_xor(acc, off);
            const int t = base + u * kStride;
            if (t <= pos) {
                acc *= scale;
                if (c == 0) s_sc[t] = acc;
                mx = fmaxf(mx, acc);
            }
        }
    }
    mx = block_max(mx, s_redf);                                          // its barriers also publish s_sc
    float zs = 0.f;
    for (int t = tid; t <= pos; t += kBlock) {
        const float p = __expf(s_sc[t] - mx);
        s_sc[t] = p;
        zs += p;
    }
    const float Z = block_sum_f32(zs, s_redf);
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
    for (int base = wave * G + g; base - g - wave * G <= pos; base += kStride * kAttnUnroll) {
        u32x4b w4[kAttnUnroll];
        float p[kAttnUnroll];
#pragma unroll
        for (int u = 0; u < kAttnUnroll; ++u) {
            const int t = base + u * kStride;
            w4[u] = *reinterpret_cast<const u32x4b*>(Vr + (size_t)min(t, pos) * d + c * 8);
            p[u] = (t <= pos) ? s_sc[t] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kAttnUnroll; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[2 * e] += p[u] * __builtin_bit_cast(float, w4[u][e] << 16);
                o[2 * e + 1] += p[u] * __builtin_bit_cast(float, w4[u][e] & 0xffff0000u);
            }
    }
#pragma unroll
    for (int off = LPK; off < kWave; off <<= 1)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += __shfl_xor(o[e], off);
    if (lane < LPK) {
#pragma unroll
        for (int e = 0; e < 8; ++e) s_part[wave][lane * 8 + e] = o[e];
    }
    __syncthreads();
    if (tid < hd) {
        const float sum = ((s_part[0][tid] + s_part[1][tid]) + (s_part[2][tid] + s_part[3][tid])) / Z;
        att[(size_t)r * d + hh * hd + tid] = f32_to_bf16_bits(sum);
    }
}

__global__ void k_body_fill_ones(float* p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 1.f;
}

__global__ void k_body_rollback(int rows, int rows_per_seq, int gamma, const int32_t* __restrict__ ctx_base,
                                const int32_t* __restrict__ accept_len, int32_t* __restrict__ ctx_len) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    const int k = accept_len[r / rows_per_seq];
    const int kept = (k + 1 < gamma) ? k + 1 : gamma;
    ctx_len[r] = ctx_base[r] + (kept < 0 ? 0 : kept);
}

// ---------------------------------------------------------------- host side
static size_t al256(size_t x) { return (x + 255) / 256 * 256; }

// A projection [rows,K] x [N,K]^T can also run as an LM head with vocabulary N, hidden size K, one draft and `rows`
// sequences: the route of shapes the split kernel does not take.
static tabed_cfg gemm_cfg(int rows, int K, int N) {
    tabed_cfg c{};
    c.V = N; c.d = K; c.n = 1; c.B = rows; c.gamma = 1; c.h = 1; c.w_dtype = 1; c.distance = 0; c.policy = 0;
    c.tau_w = 1.f; c.eps = 1e-6f; c.seed = 0;
    return c;
}

// Number of K ranges of the split kernel (0: the shape goes through the LM-head kernels instead).  Every wave gets
// the same whole number of 16-wide k-steps, at least two; the split stops growing once a launch has 256 workgroups.
static int proj_splits(int rows, int K, int N) {
    if (rows > 64 || K % 64 != 0 || N % 4 != 0) return 0;
    const int tiles = (N + 31) / 32, units = K / 64;       // a unit = one k-step for each of the four waves
    int best = 0;
    for (int ks = 1; ks <= 16; ++ks) {
        if (units % ks != 0 || units / ks < 2) continue;
        best = ks;
        if (tiles * ks >= 256) break;
    }
    return best;                                           // 0 when K == 64
}

// Chunk width (in 64s) of the wide kernel, 0 when the shape keeps to the kernel above: results of at least 2048
// columns, the widest chunk that still gives about a hundred workgroups, at most 16 ranges.
static int proj_wide_kg(int rows, int K, int N) {
    if (proj_splits(rows, K, N) == 0 || N < 2048) return 0;
    const int groups = (N + 127) / 128;
    int pick = 0;
    for (int kg = 1; kg <= 4; ++kg) {
        if (K % (kg * 64) != 0 || K / (kg * 64) > 16) continue;
        if (pick == 0 || groups * (K / (kg * 64)) >= 100) pick = kg;
    }
    return pick;
}

static int proj_slabs(int rows, int K, int N) {
    const int kg = proj_wide_kg(rows, K, N);
    if (kg != 0) return K / (kg * 64);
    const int ks = proj_splits(rows, K, N);
    return ks > 0 ? ks : 1;
}

BodyLayout body_layout(const tabed_body_cfg& c, int rows) {
    BodyLayout L;
    const int act = (c.d > c.d_ff) ? c.d : c.d_ff;
    const int shapes[4][2] = {{c.d, 3 * c.d}, {c.d, c.d}, {c.d, 2 * c.d_ff}, {c.d_ff, c.d}};   // {K, N}
    size_t ybytes = 0, g = 0;
    for (const auto& kn : shapes) {
        const int ks = proj_splits(rows, kn[0], kn[1]);
        const size_t yb = sizeof(float) * (size_t)proj_slabs(rows, kn[0], kn[1]) * rows * kn[1];
        ybytes = yb > ybytes ? yb : ybytes;
        if (ks == 0) {
            const size_t t = ws_layout(gemm_cfg(rows, kn[0], kn[1])).total;
            g = t > g ? t : g;
        }
    }
    size_t off = 0;
    L.off_ones = off; off = al256(off + sizeof(float) * (size_t)rows);
    L.off_x = off;    off = al256(off + sizeof(float) * (size_t)rows * c.d);
    L.off_y = off;    off = al256(off + ybytes);
    L.off_hb = off;   off = al256(off + sizeof(uint16_t) * (size_t)rows * act);
    L.off_gemm = off; off = al256(off + g);
    L.total = off;
    return L;
}

int validate_body_cfg(const tabed_body_cfg* c, int rows) {
    if (c == nullptr) return TABED_ENULL;
    if (c->layers < 1 || c->layers > TABED_BODY_MAX_LAYERS) return TABED_ERANGE;
    if (c->d < 8 || c->d % 8 != 0 || c->d_ff < 8 || c->d_ff % 8 != 0 || c->heads < 1 || c->d % c->heads != 0) return TABED_EINVAL;
    const int hd = c->d / c->heads;
    if (hd != 8 && hd != 16 && hd != 32 && hd != 64 && hd != 128) return TABED_EINVAL;
    if (c->V < 1 || c->max_ctx < 1 || c->max_ctx > 8192) return TABED_ERANGE;
    if (!(c->rope_theta > 0.f) || !(c->rms_eps > 0.f)) return TABED_EINVAL;
    if (rows < 1 || rows > 65535) return TABED_ERANGE;
    if (c->d > 8192 || 2 * c->d_ff > 262144) return TABED_ERANGE;      // a row of the residual stream sits in LDS
    return TABED_OK;
}

hipError_t launch_body_init(const tabed_body_cfg& c, int rows, char* ws, hipStream_t s) {
    const BodyLayout L = body_layout(c, rows);
    launch(nullptr, k_body_fill_ones, dim3((rows + 255) / 256), dim3(256), 0, s, reinterpret_cast<float*>(ws + L.off_ones), rows);
    return hipGetLastError();
}

struct Slabs {
    int ks;          // partial sums the consumer adds up
    size_t stride;   // floats between them
};

// y[ks][rows,N] = in[rows,K] x W[N,K]^T, as `ks` partial sums
static hipError_t projection(int rows, int K, int N, char* gemm_ws, const void* W, const uint16_t* in, const float* ones,
                             float* y, Slabs* out, hipStream_t s) {
    const int ks = proj_splits(rows, K, N);
    out->stride = (size_t)rows * N;
    if (ks == 0) {
        out->ks = 1;
        const tabed_cfg gc = gemm_cfg(rows, K, N);
        return launch_lmhead(gc, ws_layout(gc), gemm_ws, W, in, ones, y, s, TABED_K_BODY);
    }
    ProfScope prof(TABED_K_BODY, s);
    const uint16_t* Wb = static_cast<const uint16_t*>(W);
    const int kg = proj_wide_kg(rows, K, N);
    if (kg != 0) {
        out->ks = K / (kg * 64);
        const dim3 wgrid((N + 127) / 128, out->ks);
        const bool one = rows <= 32;
#define TABED_WIDE(KG_)                                                                                              \
    if (kg == KG_) {                                                                                                 \
        if (one) launch(&prof, k_body_proj_wide<1, KG_>, wgrid, dim3(kBlock), 0, s, rows, N, K, in, Wb, y, out->stride); \
        else     launch(&prof, k_body_proj_wide<2, KG_>, wgrid, dim3(kBlock), 0, s, rows, N, K, in, Wb, y, out->stride); \
    }
        TABED_WIDE(1) TABED_WIDE(2) TABED_WIDE(3) TABED_WIDE(4)
#undef TABED_WIDE
        return hipGetLastError();
    }
    out->ks = ks;
    const dim3 grid((N + 31) / 32, ks);
    const int steps_per_wave = K / 64 / ks;
    if (rows <= 32)
        launch(&prof, k_body_proj<1>, grid, dim3(kBlock), 0, s, rows, N, K, steps_per_wave, in, static_cast<const uint16_t*>(W), y,
               out->stride);
    else
        launch(&prof, k_body_proj<2>, grid, dim3(kBlock), 0, s, rows, N, K, steps_per_wave, in, static_cast<const uint16_t*>(W), y,
               out->stride);
    return hipGetLastError();
}

template <int LPK>
static void launch_attn(const ProfScope* prof, const tabed_body_cfg& c, int rows, Slabs sl, const float* y, const int32_t* ctx_len,
                        uint16_t* kc, uint16_t* vc, uint16_t* att, hipStream_t s) {
    launch(prof, k_body_rope_attn<LPK>, dim3(c.heads, rows), dim3(kBlock), sizeof(float) * (size_t)c.max_ctx, s, c.d, c.max_ctx,
           (double)c.rope_theta, sl.ks, sl.stride, y, ctx_len, kc, vc, att);
}

hipError_t launch_body_step(const tabed_body_cfg& c, const tabed_body_weights& w, char* ws, int rows,
                            const int32_t* token_src, int token_stride, int rows_per_token, int32_t* ctx_len,
                            uint16_t* kcache, uint16_t* vcache, uint16_t* H, hipStream_t s) {
    const BodyLayout L = body_layout(c, rows);
    const float* ones = reinterpret_cast<const float*>(ws + L.off_ones);
    float* x = reinterpret_cast<float*>(ws + L.off_x);
    float* y = reinterpret_cast<float*>(ws + L.off_y);
    uint16_t* hb = reinterpret_cast<uint16_t*>(ws + L.off_hb);
    char* gws = ws + L.off_gemm;
    const int d = c.d, hd = c.d / c.heads;
    hipError_t e;
    Slabs sl;
#define TABED_BODY_CHECK()            \
    e = hipGetLastError();            \
    if (e != hipSuccess) return e
    {
        ProfScope prof(TABED_K_BODY, s);
        launch(&prof, k_body_embed_norm, dim3(rows), dim3(kBlock), 0, s, d, c.V, c.rms_eps, token_src, token_stride,
               rows_per_token, static_cast<const uint16_t*>(w.embed), w.g_attn[0], x, hb);
        TABED_BODY_CHECK();
    }
    for (int l = 0; l < c.layers; ++l) {
        e = projection(rows, d, 3 * d, gws, w.wqkv[l], hb, ones, y, &sl, s);
        if (e != hipSuccess) return e;
        {
            ProfScope prof(TABED_K_BODY, s);
            const size_t layer_off = (size_t)l * rows * c.max_ctx * d;
            uint16_t* kc = kcache + layer_off;
            uint16_t* vc = vcache + layer_off;
            switch (hd) {
                case 8: launch_attn<1>(&prof, c, rows, sl, y, ctx_len, kc, vc, hb, s); break;
                case 16: launch_attn<2>(&prof, c, rows, sl, y, ctx_len, kc, vc, hb, s); break;
                case 32: launch_attn<4>(&prof, c, rows, sl, y, ctx_len, kc, vc, hb, s); break;
                case 64: launch_attn<8>(&prof, c, rows, sl, y, ctx_len, kc, vc, hb, s); break;
                case 128: launch_attn<16>(&prof, c, rows, sl, y, ctx_len, kc, vc, hb, s); break;
                default: return hipErrorInvalidValue;
            }
            TABED_BODY_CHECK();
        }
        e = projection(rows, d, d, gws, w.wo[l], hb, ones, y, &sl, s);
        if (e != hipSuccess) return e;
        {
            ProfScope prof(TABED_K_BODY, s);
            launch(&prof, k_body_add_norm, dim3(rows), dim3(kBlock), sizeof(float) * (size_t)d, s, d, c.rms_eps, sl.ks, sl.stride, x, y,
                   w.g_mlp[l], hb, static_cast<int32_t*>(nullptr));
            TABED_BODY_CHECK();
        }
        e = projection(rows, d, 2 * c.d_ff, gws, w.wgu[l], hb, ones, y, &sl, s);
        if (e != hipSuccess) return e;
        {
            ProfScope prof(TABED_K_BODY, s);
            const size_t count = (size_t)rows * c.d_ff;
            launch(&prof, k_body_silu_mul, dim3((unsigned)((count + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, rows, c.d_ff, sl.ks,
                   sl.stride, y, hb);
            TABED_BODY_CHECK();
        }
        e = projection(rows, c.d_ff, d, gws, w.wdown[l], hb, ones, y, &sl, s);
        if (e != hipSuccess) return e;
        {
            ProfScope prof(TABED_K_BODY, s);
            const bool last = (l + 1 == c.layers);
            launch(&prof, k_body_add_norm, dim3(rows), dim3(kBlock), sizeof(float) * (size_t)d, s, d, c.rms_eps, sl.ks, sl.stride, x, y,
                   last ? w.g_final : w.g_attn[l + 1], last ? H : hb, last ? ctx_len : static_cast<int32_t*>(nullptr));
            TABED_BODY_CHECK();
        }
    }
#undef TABED_BODY_CHECK
    return hipSuccess;
}

hipError_t launch_body_rollback(int rows, int rows_per_seq, int gamma, const int32_t* ctx_base, const int32_t* accept_len,
                                int32_t* ctx_len, hipStream_t s) {
    launch(nullptr, k_body_rollback, dim3((rows + 255) / 256), dim3(256), 0, s, rows, rows_per_seq, gamma, ctx_base, accept_len,
           ctx_len);
    return hipGetLastError();
}

}  // namespace tabed
