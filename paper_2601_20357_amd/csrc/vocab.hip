// Vocabulary-wide passes of a TABED round on gfx950: ensemble + draft token (Alg. 1 (W-Avg and Sample steps)),
// target statistics + per-draft KL + accept chain (Sec. 3 items 2-3, Sec. 5.1), corrected / bonus token
// (Sec. 3 item 3), window + weights (Alg. 1 (weight-selection step), App. B.2).  All of them are HBM- or latency-bound:
// DPP lane exchanges and a few LDS words do the reductions, fp64 carries the cross-wave and cross-workgroup
// sums, and partial results cross workgroups through device-scope atomic stores that are waited for before an
// arrival counter moves (no cache-flushing fences).
#include "device_utils.h"
#include "internal.h"

namespace tabed {

// =====================================================================================================
// Small kernels: workspace init, Philox dump, weights.
// =====================================================================================================
__global__ void k_fill_u32(uint32_t* p, int count) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0u;
}

hipError_t launch_ws_init(const tabed_cfg& c, const WsLayout& L, char* ws, hipStream_t s) {
    const int count = 5 * c.B;
    launch(nullptr, k_fill_u32, dim3((count + 255) / 256), dim3(256), 0, s,
                       reinterpret_cast<uint32_t*>(ws + L.off_tickets), count);
    return hipGetLastError();
}

__global__ void k_null() {}

hipError_t launch_null(hipStream_t s) {
    ProfScope prof(TABED_K_NULL, s);
    launch(&prof, k_null, dim3(1), dim3(64), 0, s);
    return hipGetLastError();
}

__global__ void k_philox(uint64_t seed, uint64_t round, int B, int npos, float* out) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * npos) return;
    const int b = i / npos, pos = i % npos;
    U4 r = philox4x32_10((uint32_t)round, (uint32_t)(round >> 32), (uint32_t)b, (uint32_t)pos,
                         (uint32_t)seed, (uint32_t)(seed >> 32));
    out[2 * i + 0] = u01(r.x);
    out[2 * i + 1] = u01(r.y);
}

hipError_t launch_philox(const tabed_cfg& c, uint64_t round, float* out, hipStream_t s) {
    const int count = c.B * (c.gamma + 1);
    launch(nullptr, k_philox, dim3((count + 255) / 256), dim3(256), 0, s, c.seed, round, c.B, c.gamma + 1, out);
    return hipGetLastError();
}

// Window + weights for one sequence, executed by ONE wave (64 lanes).  The window after pushing the nv new
// positions is the newest min(count + nv, h) entries of (old ring entries ++ new entries); every lane loads
// its share of them in parallel (no load depends on a store), lane j sums column j in fp64, the policy
// follows (softmax of 1/e over the n drafts, or arg-min over the 11 candidate mixtures), and only then are the
// new positions stored into the ring.  h = 0 (window ALL): one running fp32 sum per column.  dw = width of
// one distance vector.  PUB: the distances were just published by another workgroup of the same kernel and
// must be read at device scope.  Lanes exchange through two small LDS arrays; LDS operations of one wave
// execute in order, so no barrier is involved.  A few hundred scalars: latency-bound.
struct WindowArgs {
    int n, dw, gamma, h, policy;
    double tau_w, eps;
    uint64_t seed, round;   // policy 3: Philox key and the round the weights are for
    float* ring;
    int32_t* ring_head;
    int32_t* ring_count;
    float* weights;
};

template <bool PUB>
__device__ __forceinline__ float dev_load(const float* p) { return PUB ? published_load(p) : *p; }

template <bool PUB>
__device__ __forceinline__ void window_update(const WindowArgs& a, int b, int lane, const float* dev, int nv,
                                              double* s_part /* [64] */, double* s_x /* [TABED_MAX_N] */) {
    const int n = a.n, dw = a.dw, gamma = a.gamma, h = a.h, policy = a.policy;
    nv = (dev == nullptr) ? 0 : (nv < 0 ? 0 : (nv > gamma ? gamma : nv));
    const float* db = dev ? dev + (size_t)b * gamma * dw : nullptr;
    bool empty;
    if (h == 0) {
        int count = a.ring_count[b];
        count = count < 0 ? 0 : count;
        if (lane < dw) {
            float sum = a.ring[(size_t)b * dw + lane];
            for (int i = 0; i < nv; ++i) sum = sum + dev_load<PUB>(db + (size_t)i * dw + lane);   // fp32, in order
            if (nv > 0) a.ring[(size_t)b * dw + lane] = sum;
            s_x[lane] = (policy == 2) ? (double)sum : (1.0 / fmax((double)sum, a.eps)) / a.tau_w;
        }
        const long long total = (long long)count + nv;
        if (lane == 0 && nv > 0) a.ring_count[b] = total > 0x7fffffffLL ? 0x7fffffff : (int)total;
        empty = (total == 0);
    } else {
        int head = a.ring_head[b], count = a.ring_count[b];
        head = ((head % h) + h) % h;
        count = count < 0 ? 0 : (count > h ? h : count);
        const int new_count = (count + nv < h) ? count + nv : h;
        float* rb = a.ring + (size_t)b * h * dw;
        const int per = 64 / dw;                      // lanes per column (dw <= 16 => per >= 4)
        const int j = lane % dw, t0 = lane / dw;
        double acc = 0.0;
        if (lane < per * dw) {
            for (int r = t0; r < new_count; r += per) {   // r-th newest entry of the new window
                float v;
                if (r < nv) v = dev_load<PUB>(db + (size_t)(nv - 1 - r) * dw + j);
                else        v = rb[(size_t)((((head - 1 - (r - nv)) % h) + h) % h) * dw + j];
                acc += (double)v;
            }
        }
        s_part[lane] = acc;
        __builtin_amdgcn_wave_barrier();
        if (lane < dw) {
            double e = 0.0;
            for (int q = 0; q < per; ++q) e += s_part[q * dw + lane];
            s_x[lane] = (policy == 2) ? e : (1.0 / fmax(e, a.eps)) / a.tau_w;
        }
        if (nv > 0) {                                 // all window loads above are complete: store the new entries
            for (int idx = lane; idx < nv * dw; idx += 64) {
                const int i = idx / dw, jj = idx % dw;
                if (i >= nv - h) rb[(size_t)((head + i) % h) * dw + jj] = dev_load<PUB>(db + (size_t)i * dw + jj);
            }
            if (lane == 0) {
                a.ring_head[b] = (head + nv) % h;
                a.ring_count[b] = new_count;
            }
        }
        empty = (new_count == 0);
    }
    if (policy == 3 && lane < n) {                     // random weights: E_j = -ln U_j, normalised below
        const U4 r = philox4x32_10((uint32_t)a.round, (uint32_t)(a.round >> 32), (uint32_t)b,
                                   (uint32_t)(gamma + 1 + lane / 4), (uint32_t)a.seed, (uint32_t)(a.seed >> 32));
        const uint32_t x = (lane & 3) == 0 ? r.x : (lane & 3) == 1 ? r.y : (lane & 3) == 2 ? r.z : r.w;
        s_x[lane] = -log(((double)(x >> 8) + 0.5) * (1.0 / 16777216.0));
    }
    __builtin_amdgcn_wave_barrier();
    if (lane < n) {
        float w;
        if (policy == 3) {
            double tot = 0.0;
            for (int q = 0; q < n; ++q) tot += s_x[q];
            w = (float)(s_x[lane] / tot);
        } else if (policy == 1 || empty) {
            w = (float)(1.0 / (double)n);
        } else if (policy == 2) {
            int best = 0;                             // arg-min of the window sums, lowest index on ties
            for (int q = 1; q < dw; ++q) if (s_x[q] < s_x[best]) best = q;
            const double w1 = (double)best / (double)(dw - 1);
            w = (float)(lane == 0 ? 1.0 - w1 : w1);
        } else {
            double xmax = -INFINITY;
            for (int q = 0; q < n; ++q) xmax = fmax(xmax, s_x[q]);
            double Z = 0.0;
            for (int q = 0; q < n; ++q) Z += exp(s_x[q] - xmax);
            w = (float)(exp(s_x[lane] - xmax) / Z);
        }
        if (PUB) publish_store(&a.weights[(size_t)b * n + lane], w);
        else a.weights[(size_t)b * n + lane] = w;
    }
}

__global__ __launch_bounds__(64) void k_weights(WindowArgs a, const float* __restrict__ dev,
                                                const int32_t* __restrict__ n_valid) {
    __shared__ double s_part[64];
    __shared__ double s_x[TABED_MAX_N];
    const int b = blockIdx.x;
    const int nv = (dev != nullptr && n_valid != nullptr) ? n_valid[b] : 0;
    window_update<false>(a, b, threadIdx.x, (dev != nullptr && n_valid != nullptr) ? dev : nullptr, nv, s_part, s_x);
}

static WindowArgs window_args(const tabed_cfg& c, uint64_t round, float* ring, int32_t* ring_head, int32_t* ring_count,
                              float* weights) {
    WindowArgs a;
    a.seed = c.seed; a.round = round;
    a.n = c.n; a.dw = (c.policy == 2) ? TABED_GRID_CANDIDATES : c.n; a.gamma = c.gamma; a.h = c.h; a.policy = c.policy;
    a.tau_w = (double)c.tau_w; a.eps = (double)c.eps;
    a.ring = ring; a.ring_head = ring_head; a.ring_count = ring_count; a.weights = weights;
    return a;
}

hipError_t launch_weights(const tabed_cfg& c, uint64_t round, const float* dev, const int32_t* n_valid, float* ring,
                          int32_t* ring_head, int32_t* ring_count, float* weights, hipStream_t s) {
    ProfScope prof(TABED_K_WEIGHTS, s);
    launch(&prof, k_weights, dim3(c.B), dim3(64), 0, s, window_args(c, round, ring, ring_head, ring_count, weights), dev,
           n_valid);
    return hipGetLastError();
}

// =====================================================================================================
// Ensemble + draft token.
// The LM-head epilogue left, per draft row and per 32-wide vocabulary tile, the tile maximum of the scaled
// logits and the tile sum of exp(scaled logit - tile maximum).  From those alone this kernel gets every
// draft's log-sum-exp and the mass of the mixture q = sum_j w_j q^(j) inside every tile; a sampling row
// therefore reads logits only inside the one tile its uniform falls into.  Every thread loads the partials
// of its own tiles (all drafts) in one burst of independent loads and keeps them in registers, so the kernel
// pays two memory round trips (partials, then the chosen tile) instead of one per reduction.  A greedy row needs
// the arg-max of q over the whole vocabulary: its row is split over gridDim.x workgroups and the last one
// to arrive merges the candidates (lowest index wins ties, so arrival order does not matter).
// =====================================================================================================
struct SampleArgs {
    int V, n, B, gamma, pos, NT, C2;
    int sib, S;           // token tree: sibling index of this launch (0 = the trunk token) and siblings per position
    const int32_t* trunk; // token tree, sib > 0: trunk tokens [B,gamma] (a greedy row's siblings skip taken tokens)
    uint64_t seed, round;
    const float* logits;  // [B,n,V] of this position
    const float* pm;      // [B*n,NT]
    const float* ps;      // [B*n,NT]
    const float* weights;
    const float* temperature;
    const float* u_draft;
    double* draft_lse;
    int32_t* draft_tokens;
    float* draft_q;
    uint8_t* flags;
    Top2Rec* cand;
    uint32_t* tickets;
};

// TI = tiles per thread, a compile-time bound with NT <= kBlock * TI, so that every phase issues all of its
// loads before the first use and keeps its tile values in registers.  N = number of drafts when it is known
// at compile time (0 = run time): then the partials are read ONCE, each thread keeping the n*TI terms
// ps*exp(pm - m_j) of its own run of tiles in registers for both the log-sum-exp and the tile masses.
template <bool VEC, int TI, int N>
__global__ __launch_bounds__(kBlock) void k_sample(SampleArgs a) {
    const int b = blockIdx.y, c = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = (N > 0) ? N : a.n, NT = a.NT, V = a.V;
    // Workgroup 0 of a sequence always has work, so its temperature load overlaps the loads below; the
    // other workgroups only exist for greedy rows and leave at once otherwise.
    const float T = a.temperature[b];
    if (c != 0 && T > 0.f) return;

    __shared__ float s_m[TABED_MAX_N];    // row maximum of scaled logits
    __shared__ double s_S[TABED_MAX_N];   // sum_v exp(scaled - max)
    __shared__ double s_c[TABED_MAX_N];   // w_j / S_j
    __shared__ float s_cf[TABED_MAX_N];
    __shared__ int s_first[kWavesPerBlock], s_lastw[kWavesPerBlock], s_tile, s_last;
    __shared__ double s_prefix;
    __shared__ Top2 s_top[kWavesPerBlock];
    __shared__ double s_term[TABED_MAX_N][kTileV];
    __shared__ float s_wm[kWavesPerBlock][TABED_MAX_N];
    __shared__ double s_wsum[kWavesPerBlock][TABED_MAX_N];
    __shared__ double s_wtot[kWavesPerBlock][5];        // wave totals of the tile-mass scan, per chunk row

    const float* pmb = a.pm + (size_t)b * n * NT;      // partials of this sequence: [n][NT]
    const float* psb = a.ps + (size_t)b * n * NT;
    // the trunk token goes to [B,gamma]; sibling s of a token tree to [B,gamma,S] and has a Philox block of its own
    const size_t out_idx = (a.sib == 0) ? (size_t)b * a.gamma + a.pos
                                        : ((size_t)b * a.gamma + a.pos) * a.S + (a.sib - 1);
    const float wj = (tid < n) ? a.weights[(size_t)b * n + tid] : 0.f;
    const float u = a.u_draft ? a.u_draft[out_idx]
                              : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)a.pos + (uint32_t)a.sib * kSiblingStride, 0);
    int taken[TABED_MAX_TREE_WIDTH - 1];               // greedy siblings: tokens already in the candidate list
#pragma unroll
    for (int t = 0; t < TABED_MAX_TREE_WIDTH - 1; ++t) taken[t] = -1;
    if (a.sib > 0) {
        taken[0] = a.trunk[(size_t)b * a.gamma + a.pos];
#pragma unroll
        for (int t = 1; t < TABED_MAX_TREE_WIDTH - 1; ++t)
            if (t < a.sib) taken[t] = a.draft_tokens[((size_t)b * a.gamma + a.pos) * a.S + (t - 1)];
    }

    // Which tiles a thread owns.  Two-pass kernels and TI = 1: the contiguous run [tid*TI, tid*TI + TI).
    // Single-pass kernels: TI/4 chunks of 4 consecutive tiles, chunk q*256 + tid for q < TI/4 (for TI = 4 that
    // is the same run) -- every load is then 16 bytes and a wave's load is one contiguous kilobyte.
    constexpr bool CHUNKED = (N > 0 && TI >= 4);
    constexpr int TPC = CHUNKED ? 4 : TI;              // tiles per chunk
    constexpr int Q = TI / TPC;                        // chunks per thread
    auto tile_of = [&](int i) { return CHUNKED ? ((i / 4) * kBlock + tid) * 4 + (i & 3) : tid * TI + i; };

    float uu[(N > 0) ? N : 1][TI];                     // single pass: terms of this thread's tiles, all drafts
    double lse_mine = 0.0;
    if (N > 0) {
        // ---- single pass over the partials of every draft
        float pmv[(N > 0) ? N : 1][TI], psv[(N > 0) ? N : 1][TI];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            if (CHUNKED && (NT & 3) == 0) {
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const int t = tile_of(4 * q);
                    float4 m4 = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY), s4 = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (t < NT) {
                        m4 = *reinterpret_cast<const float4*>(pmb + (size_t)j * NT + t);
                        s4 = *reinterpret_cast<const float4*>(psb + (size_t)j * NT + t);
                    }
                    pmv[j][4 * q] = m4.x; pmv[j][4 * q + 1] = m4.y; pmv[j][4 * q + 2] = m4.z; pmv[j][4 * q + 3] = m4.w;
                    psv[j][4 * q] = s4.x; psv[j][4 * q + 1] = s4.y; psv[j][4 * q + 2] = s4.z; psv[j][4 * q + 3] = s4.w;
                }
            } else {
#pragma unroll
                for (int i = 0; i < TI; ++i) {
                    const int t = tile_of(i);
                    pmv[j][i] = t < NT ? pmb[(size_t)j * NT + t] : -INFINITY;
                    psv[j][i] = t < NT ? psb[(size_t)j * NT + t] : 0.f;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < N; ++j) {
            float ml = -INFINITY;
#pragma unroll
            for (int i = 0; i < TI; ++i) ml = fmaxf(ml, pmv[j][i]);
            ml = wave_max(ml);
            if (lane == 0) s_wm[wave][j] = ml;
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const float M = fmaxf(fmaxf(s_wm[0][j], s_wm[1][j]), fmaxf(s_wm[2][j], s_wm[3][j]));
            float sl = 0.f;
#pragma unroll
            for (int i = 0; i < TI; ++i) {
                uu[j][i] = (psv[j][i] > 0.f) ? psv[j][i] * __expf(pmv[j][i] - M) : 0.f;
                sl += uu[j][i];
            }
            const double S = (double)wave_sum(sl);         // 64 x TI terms in fp32, fp64 across the four waves
            if (lane == 0) s_wsum[wave][j] = S;
        }
        __syncthreads();
        if (tid < N) {                                     // thread j: everything the later phases need of draft j
            const int j = tid;
            const float M = fmaxf(fmaxf(s_wm[0][j], s_wm[1][j]), fmaxf(s_wm[2][j], s_wm[3][j]));
            const double S = (s_wsum[0][j] + s_wsum[1][j]) + (s_wsum[2][j] + s_wsum[3][j]);
            s_m[j] = M;
            s_S[j] = S;
            s_c[j] = (double)wj / S;
            s_cf[j] = (float)s_c[j];
            lse_mine = (double)M + log(S);                 // stored after the barrier below
        }
    } else {
        // ---- per-draft log-sum-exp: one wave per draft row, lanes strided over the row's tiles
        constexpr int TL = TI * kWavesPerBlock;        // tiles per lane when one wave covers a whole row
        for (int j = wave; j < n; j += kWavesPerBlock) {
            float pmv[TL], psv[TL];
#pragma unroll
            for (int i = 0; i < TL; ++i) {
                const int t = lane + i * kWave;
                pmv[i] = t < NT ? pmb[(size_t)j * NT + t] : -INFINITY;
                psv[i] = t < NT ? psb[(size_t)j * NT + t] : 0.f;
            }
            float ml = -INFINITY;
#pragma unroll
            for (int i = 0; i < TL; ++i) ml = fmaxf(ml, pmv[i]);
            const float M = wave_max(ml);
            float sl = 0.f;
#pragma unroll
            for (int i = 0; i < TL; ++i) sl += (psv[i] > 0.f) ? psv[i] * __expf(pmv[i] - M) : 0.f;
            const double S = wave_sum((double)sl);
            if (lane == 0) {
                s_m[j] = M;
                s_S[j] = S;
                if (c == 0 && a.sib == 0) a.draft_lse[((size_t)a.pos * a.B + b) * n + j] = (double)M + log(S);
            }
        }
    }
    const bool greedy = !(T > 0.f);
    const float invT = greedy ? 1.f : 1.f / T;
    __syncthreads();
    if (N > 0) {
        if (tid < N && c == 0 && a.sib == 0) a.draft_lse[((size_t)a.pos * a.B + b) * n + tid] = lse_mine;
    } else {
        if (tid < n) {
            s_c[tid] = (double)wj / s_S[tid];
            s_cf[tid] = (float)s_c[tid];
        }
        __syncthreads();
    }

    const float* rows = a.logits + (size_t)b * n * V;

    if (!greedy) {
        // ---- tile masses of the mixture: thread tid owns tiles [tid*TI, tid*TI + TI), kept in registers
        double mt[TI];
#pragma unroll
        for (int i = 0; i < TI; ++i) mt[i] = 0.0;
        double Z = 0.0;
        if (N > 0) {
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const double cj = s_c[j];
                Z += cj * s_S[j];
#pragma unroll
                for (int i = 0; i < TI; ++i) mt[i] += cj * (double)uu[j][i];
            }
        } else {
#pragma unroll 4
            for (int j = 0; j < n; ++j) {
                float pmv[TI], psv[TI];
#pragma unroll
                for (int i = 0; i < TI; ++i) {
                    const int t = tile_of(i);
                    pmv[i] = t < NT ? pmb[(size_t)j * NT + t] : -INFINITY;
                    psv[i] = t < NT ? psb[(size_t)j * NT + t] : 0.f;
                }
                const double cj = s_c[j];
                const float mj = s_m[j];
                Z += cj * s_S[j];
#pragma unroll
                for (int i = 0; i < TI; ++i)
                    if (psv[i] > 0.f) mt[i] += cj * (double)(psv[i] * __expf(pmv[i] - mj));
            }
        }
        // ---- prefix over the tile masses in tile order.  Chunk q of thread tid has key q*256 + tid; keys
        //      order the chunks along the vocabulary.  One wave scan per chunk row, one barrier.
        double cs[Q], cinc[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            cs[q] = 0.0;
#pragma unroll
            for (int e = 0; e < TPC; ++e) cs[q] += mt[q * TPC + e];
            cinc[q] = wave_inclusive_scan(cs[q]);
            if (lane == 63) s_wtot[wave][q] = cinc[q];
        }
        __syncthreads();
        const double target = (double)u * Z;
        double excl[Q];
        int first_key = 0x7fffffff, last_key = -1;
        {
            double rowbase = 0.0;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                double before = rowbase;
                for (int w = 0; w < wave; ++w) before += s_wtot[w][q];
                excl[q] = before + (cinc[q] - cs[q]);
                if (cs[q] > 0.0) {
                    if (first_key == 0x7fffffff && excl[q] + cs[q] > target) first_key = q * kBlock + tid;
                    last_key = q * kBlock + tid;
                }
                rowbase += ((s_wtot[0][q] + s_wtot[1][q]) + s_wtot[2][q]) + s_wtot[3][q];
            }
        }
        const int key = block_pick_key(first_key, last_key, s_first, s_lastw);   // -1 only if every mass is zero
        if (key < 0) {
            if (tid == 0) {
                a.draft_tokens[out_idx] = 0;
                a.draft_q[out_idx] = 0.f;
                a.flags[out_idx] = (uint8_t)(TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE);
            }
            return;
        }
        if (tid == (key & (kBlock - 1))) {
            const int qs = key / kBlock;
            double P = 0.0, Plast = 0.0;
            int istar = -1, ilast = 0;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (q == qs) {
                    P = excl[q]; Plast = P; ilast = q * TPC;
#pragma unroll
                    for (int e = 0; e < TPC; ++e) {
                        const int i = q * TPC + e;
                        if (istar < 0) {
                            if (mt[i] > 0.0) { ilast = i; Plast = P; }
                            if (P + mt[i] > target) istar = i;
                            else P += mt[i];
                        }
                    }
                }
            }
            if (istar < 0) { istar = ilast; P = Plast; }
            s_tile = tile_of(istar);
            s_prefix = P;
        }
        __syncthreads();
        // ---- the tile's logits: thread (draft j, lane v) -> one round trip for all drafts, summed by wave 0
        {
            const int vl = tid & (kTileV - 1), v = s_tile * kTileV + vl;
            for (int j = tid / kTileV; j < n; j += kBlock / kTileV)
                s_term[j][vl] = (v < V) ? s_c[j] * (double)__expf(rows[(size_t)j * V + v] * invT - s_m[j]) : 0.0;
        }
        __syncthreads();
        if (tid >= kWave) return;
        const int v = s_tile * kTileV + lane;
        double f = 0.0;
        if (lane < kTileV)
            for (int j = 0; j < n; ++j) f += s_term[j][lane];
        const double inc = wave_inclusive_scan(f);
        const double cdf = s_prefix + inc;
        const unsigned long long cross = __ballot(cdf > target && f > 0.0);
        const unsigned long long live = __ballot(f > 0.0);
        int pick;
        uint32_t flag = 0;
        if (cross) pick = __ffsll((long long)cross) - 1;
        else if (live) { pick = 63 - __clzll((long long)live); flag = TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE; }
        else { pick = 0; flag = TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE; }
        if (lane == pick) {
            const double tol = (double)kMargin * Z;
            if (fabs(cdf - target) < tol && v + 1 < V) flag |= TABED_FLAG_SAMPLE_MARGIN;
            if (v > 0 && fabs((cdf - f) - target) < tol) flag |= TABED_FLAG_SAMPLE_MARGIN;
            a.draft_tokens[out_idx] = v < V ? v : V - 1;
            a.draft_q[out_idx] = (float)f;
            a.flags[out_idx] = (uint8_t)flag;
        }
        return;
    }

    // ---- greedy row: arg-max (with runner-up) of the mixture over this workgroup's chunk
    // (at most kMaxGreedyChunks workgroups per row: every one of them repeats the log-sum-exp pass over the
    // row's partials, so a large vocabulary is walked in several 4096-wide strides per workgroup instead)
    Top2 best = top2_empty();
    for (int cb = c * kChunkV; cb < V; cb += a.C2 * kChunkV) {
        float q[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) q[u][e] = 0.f;
        for (int j = 0; j < n; ++j) {                      // the four loads of a draft row go out together
            float4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) x[u] = load4<VEC>(rows + (size_t)j * V, cb + (u * kBlock + tid) * 4, V);
            const float cj = s_cf[j], mj = s_m[j];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) q[u][e] += cj * __expf(f4get(x[u], e) * invT - mj);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int v = cb + (u * kBlock + tid) * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                bool free_tok = (v + e < V);
#pragma unroll
                for (int t = 0; t < TABED_MAX_TREE_WIDTH - 1; ++t) free_tok = free_tok && (v + e != taken[t]);
                if (free_tok) best = top2_push(best, q[u][e], v + e);
            }
        }
    }
    best = wave_top2(best);
    if (lane == 0) s_top[wave] = best;
    __syncthreads();
    if (tid == 0) {
        Top2 t = s_top[0];
        for (int w = 1; w < kWavesPerBlock; ++w) t = top2_merge(t, s_top[w]);
        Top2Rec* rec = &a.cand[(size_t)b * a.C2 + c];
        publish_store(&rec->v1, t.v1);
        publish_store(&rec->i1, t.i1);
        publish_store(&rec->v2, t.v2);
    }
    publish_barrier();                                     // the candidate's stores are acknowledged
    if (tid == 0) s_last = arrive(&a.tickets[b], (uint32_t)a.C2) ? 1 : 0;
    __syncthreads();
    if (!s_last || tid >= kWave) return;
    Top2 t = top2_empty();
    for (int cc = lane; cc < a.C2; cc += kWave) {
        const Top2Rec* r = &a.cand[(size_t)b * a.C2 + cc];
        t = top2_merge(t, Top2{published_load(&r->v1), published_load(&r->i1), published_load(&r->v2)});
    }
    t = wave_top2(t);
    if (lane != 0) return;
    const int y = (t.i1 >= 0 && t.i1 < V) ? t.i1 : 0;
    double f = 0.0;
    for (int j = 0; j < n; ++j) f += s_c[j] * (double)__expf(rows[(size_t)j * V + y] * invT - s_m[j]);
    uint32_t flag = 0;
    if (V > 1 + a.sib && (t.v1 - t.v2) < kMargin * fabsf(t.v1)) flag |= TABED_FLAG_SAMPLE_MARGIN;
    a.draft_tokens[out_idx] = y;
    a.draft_q[out_idx] = (float)f;
    a.flags[out_idx] = (uint8_t)flag;
}

// sib = 0: the trunk token of Alg. 1 (Sample step).  sib >= 1 (token tree of `width`): sibling `sib` of the position, from
// the same softmax partials; the output arrays are then the [B,gamma,width-1] sibling arrays.
static hipError_t launch_sample_any(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round, int pos,
                                    const float* logits, const float* weights, const float* temperature,
                                    const float* u_draft, double* draft_lse, int32_t* draft_tokens, float* draft_q,
                                    uint8_t* flags, int sib, int width, const int32_t* trunk, hipStream_t s) {
    ProfScope prof(TABED_K_SAMPLE, s);
    SampleArgs a;
    a.V = c.V; a.n = c.n; a.B = c.B; a.gamma = c.gamma; a.pos = pos; a.NT = L.NT; a.C2 = L.C2;
    a.sib = sib; a.S = width - 1; a.trunk = trunk;
    a.seed = c.seed; a.round = round;
    a.logits = logits;
    a.pm = reinterpret_cast<const float*>(ws + L.off_pm);
    a.ps = reinterpret_cast<const float*>(ws + L.off_ps);
    a.weights = weights; a.temperature = temperature; a.u_draft = u_draft;
    a.draft_lse = draft_lse; a.draft_tokens = draft_tokens; a.draft_q = draft_q; a.flags = flags;
    a.cand = reinterpret_cast<Top2Rec*>(ws + L.off_cand);
    a.tickets = reinterpret_cast<uint32_t*>(ws + L.off_tickets) + 0 * c.B;
    const dim3 grid(L.C2, c.B);
    const bool vec = (c.V % 4 == 0);
    const int ti = (L.NT + kBlock - 1) / kBlock;
    // single-pass instantiations: compile-time draft counts whose n*TI terms (x3 registers) fit a 512-register wave
    const bool ncomp_ok = vec && ti <= 20 && (c.n == 1 || c.n == 2 || c.n == 4 || (c.n == 8 && ti <= 8));
    const int nc = ncomp_ok ? c.n : 0;
#define TABED_LAUNCH_SAMPLE_N(TI_, N_) launch(&prof, k_sample<true, TI_, N_>, grid, dim3(kBlock), 0, s, a)
#define TABED_LAUNCH_SAMPLE(TI_, ALLOW8_)                                                         \
    do {                                                                                          \
        if (!vec) launch(&prof, k_sample<false, TI_, 0>, grid, dim3(kBlock), 0, s, a);            \
        else if (nc == 1) TABED_LAUNCH_SAMPLE_N(TI_, 1);                                          \
        else if (nc == 2) TABED_LAUNCH_SAMPLE_N(TI_, 2);                                          \
        else if (nc == 4) TABED_LAUNCH_SAMPLE_N(TI_, 4);                                          \
        else if (nc == 8 && ALLOW8_) TABED_LAUNCH_SAMPLE_N(TI_, (ALLOW8_ ? 8 : 1));               \
        else TABED_LAUNCH_SAMPLE_N(TI_, 0);                                                       \
    } while (0)
    if (ti <= 1) TABED_LAUNCH_SAMPLE(1, true);
    else if (ti <= 4) TABED_LAUNCH_SAMPLE(4, true);
    else if (ti <= 8) TABED_LAUNCH_SAMPLE(8, true);
    else if (ti <= 20) TABED_LAUNCH_SAMPLE(20, false);
    else if (ti <= 32) { if (vec) TABED_LAUNCH_SAMPLE_N(32, 0); else launch(&prof, k_sample<false, 32, 0>, grid, dim3(kBlock), 0, s, a); }
    else return hipErrorInvalidValue;              // V > 262144: validate_cfg rejects it before this point
#undef TABED_LAUNCH_SAMPLE_N
#undef TABED_LAUNCH_SAMPLE
    return hipGetLastError();
}

hipError_t launch_sample(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round, int pos,
                         const float* logits, const float* weights, const float* temperature,
                         const float* u_draft, double* draft_lse, int32_t* draft_tokens, float* draft_q,
                         uint8_t* flags, hipStream_t s) {
    return launch_sample_any(c, L, ws, round, pos, logits, weights, temperature, u_draft, draft_lse, draft_tokens,
                             draft_q, flags, 0, 1, nullptr, s);
}

// Token tree: the width-1 siblings of position pos, one sampler launch each (a greedy row's sibling s needs
// siblings 1..s-1 to skip them).  Uses the softmax partials the LM head of this position left in the workspace.
hipError_t launch_siblings(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round, int pos, int width,
                           const float* logits, const int32_t* draft_tokens, const float* weights,
                           const float* temperature, const float* u_sib, int32_t* sib_tokens, float* sib_q,
                           uint8_t* sib_flags, hipStream_t s) {
    for (int sib = 1; sib < width; ++sib) {
        const hipError_t e = launch_sample_any(c, L, ws, round, pos, logits, weights, temperature, u_sib, nullptr,
                                               sib_tokens, sib_q, sib_flags, sib, width, draft_tokens, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// =====================================================================================================
// Target statistics and per-draft KL sums.
// Grid (chunk, position i <= gamma, sequence b).  Each workgroup reads its chunk of the target row once,
// and for i < gamma the same chunk of the n draft rows once -- all loads issued before the first use --
// and leaves a record
//   { m_c = max scaled target logit, Z_c = sum exp(st - m_c), arg-max of the raw row,
//     A_jc = sum exp(st - m_c) * (st - s_j)  for every draft j }.
// Since KL(p || q_j) = sum_v p (st - s_j) - lse_p + lse_j, the records of a row combine exactly (fp64, chunk
// order) in the kernel that follows.  N is the number of drafts when known at compile time (0 = run time).
// Two-draft grid policy with KL: the same pass leaves, instead of the A_jc, the sums of the 11 candidate mixtures
//   A_kc = sum exp(st - m_c) * (st - log mix_k),   mix_k = (1 - k/10) q_1 + (k/10) q_2,   KL(p || mix_k) = A_k / Z - lse_p,
// so that the distances of that policy cost no pass of their own either.
// =====================================================================================================
struct StatsArgs {
    int V, n, B, gamma, C3, RS;
    int with_drafts;      // 0: only the target-row part of the records (distances come from k_dist)
    int grid;             // 1 (two drafts): the A sums are those of the 11 candidate mixtures, not of the drafts
    const float* target;
    const float* dlogits;
    const double* dlse;   // [gamma,B,n]; read only for the mixtures
    const float* temperature;
    double* stats;
};

template <bool VEC, int U, int N>
__global__ __launch_bounds__(kBlock) void k_stats(StatsArgs a) {
    const int c = blockIdx.x, i = blockIdx.y, b = blockIdx.z, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = a.V, n = (N > 0) ? N : a.n, gamma = a.gamma;
    const float T = a.temperature[b];
    const float invT = (T > 0.f) ? 1.f / T : 1.f;

    __shared__ float s_redf[kWavesPerBlock];
    __shared__ double s_redd[kWavesPerBlock];
    __shared__ ArgMax s_am[kWavesPerBlock];
    __shared__ double s_A[kWavesPerBlock][TABED_MAX_N];
    __shared__ float s_qhi[2], s_qoml[2];                // the two drafts' log-sum-exp as fp32 head + (1 - tail)

    const float* trow = a.target + ((size_t)b * (gamma + 1) + i) * V;
    const float* qbase = a.dlogits + (((size_t)i * a.B + b) * n) * V;   // only dereferenced when i < gamma
    const int cb = c * (kBlock * 4 * U);
    const bool drafts = (i < gamma) && a.with_drafts;
    const bool grid = (N == 2) && drafts && a.grid;
    if (N == 2 && grid && tid < 2) {                     // published by the barriers of the maximum below
        const double l = a.dlse[((size_t)i * a.B + b) * 2 + tid];
        const float hi = (float)l;
        s_qhi[tid] = hi;
        s_qoml[tid] = (float)(1.0 - (l - (double)hi));
    }

    float4 tx[U];
    float4 dx[(N > 0) ? N : 1][U];
#pragma unroll
    for (int u = 0; u < U; ++u) tx[u] = load4<VEC>(trow, cb + (u * kBlock + tid) * 4, V);
    if (N > 0 && drafts) {
#pragma unroll
        for (int j = 0; j < N; ++j)
#pragma unroll
            for (int u = 0; u < U; ++u) dx[j][u] = load4<VEC>(qbase + (size_t)j * V, cb + (u * kBlock + tid) * 4, V);
    }

    float st[U * 4], ex[U * 4];
    ArgMax am{-INFINITY, 0x7fffffff};
    float tmax = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int v = cb + (u * kBlock + tid) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float xe = f4get(tx[u], e);
            if (v + e < V) am = argmax_merge(am, ArgMax{xe, v + e});
            st[u * 4 + e] = xe * invT;
            tmax = fmaxf(tmax, st[u * 4 + e]);
        }
    }
    const float mc = block_max(tmax, s_redf);
    float zf = 0.f;
#pragma unroll
    for (int k = 0; k < U * 4; ++k) {
        ex[k] = (st[k] > -INFINITY) ? __expf(st[k] - mc) : 0.f;
        zf += ex[k];
    }
    const double Zw = wave_sum((double)zf);
    if (lane == 0) s_redd[wave] = Zw;
    am = wave_argmax(am);
    if (lane == 0) s_am[wave] = am;

    if (N == 2 && grid) {
        // both drafts' probabilities of this thread's elements, then one candidate mixture at a time.  The sums are
        // taken about the chunk maximum (st - m_c <= 0 where exp(st - m_c) matters) and m_c Z_c is added back in
        // fp64 when the record is written.  Bare v_log_f32 (log2): its ~1e-7 relative error is random per element
        // and averages out under the sum; a mixture below the normal range only occurs where p is negligible too.
        float q0[U * 4], q1[U * 4];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a0 = f4get(dx[0][u], e), a1 = f4get(dx[(N > 1) ? 1 : 0][u], e);
                const float p0 = (a0 > -INFINITY) ? __expf(a0 * invT - s_qhi[0]) * s_qoml[0] : 0.f;
                const float p1 = (a1 > -INFINITY) ? __expf(a1 * invT - s_qhi[1]) * s_qoml[1] : 0.f;
                q0[u * 4 + e] = p0;
                q1[u * 4 + e] = p1;
            }
        constexpr int NC = TABED_GRID_CANDIDATES;
        float tl[U * 4];                                   // log2 of exp(st - m_c), shared by the candidates
#pragma unroll
        for (int x = 0; x < U * 4; ++x) tl[x] = (ex[x] > 0.f) ? (st[x] - mc) * 1.44269504f : 0.f;
#pragma unroll
        for (int k = 0; k < NC; ++k) {
            const float w1 = (float)k / (float)(NC - 1), w0 = 1.f - w1;
            float acc = 0.f;
#pragma unroll
            for (int x = 0; x < U * 4; ++x)                // a term with p = 0 is 0 (tl is 0 there and the logarithm finite)
                acc += ex[x] * (tl[x] - __builtin_amdgcn_logf(fmaxf(fmaf(w1, q1[x], w0 * q0[x]), 1e-37f)));
            const double Ak = wave_sum((double)(acc * 0.693147181f));
            if (lane == 0) s_A[wave][k] = Ak;
        }
    } else if (drafts) {
        if (N > 0) {
#pragma unroll
            for (int j = 0; j < N; ++j) {
                float aj = 0.f;
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p = ex[u * 4 + e];
                        if (p > 0.f) aj += p * (st[u * 4 + e] - f4get(dx[j][u], e) * invT);
                    }
                const double Aj = wave_sum((double)aj);
                if (lane == 0) s_A[wave][j] = Aj;
            }
        } else {
            for (int j = 0; j < n; ++j) {
                float aj = 0.f;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int v = cb + (u * kBlock + tid) * 4;
                    const float4 y = load4<VEC>(qbase + (size_t)j * V, v, V);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p = ex[u * 4 + e];
                        if (p > 0.f) aj += p * (st[u * 4 + e] - f4get(y, e) * invT);
                    }
                }
                const double Aj = wave_sum((double)aj);
                if (lane == 0) s_A[wave][j] = Aj;
            }
        }
    }
    __syncthreads();
    double* rec = a.stats + (((size_t)b * (gamma + 1) + i) * a.C3 + c) * a.RS;
    if (tid == 0) {
        ArgMax t = s_am[0];
        for (int w = 1; w < kWavesPerBlock; ++w) t = argmax_merge(t, s_am[w]);
        rec[0] = (double)mc;
        rec[1] = (s_redd[0] + s_redd[1]) + (s_redd[2] + s_redd[3]);
        rec[2] = (double)t.v;
        rec[3] = (double)t.i;
    }
    if (grid) {
        if (tid < TABED_GRID_CANDIDATES)
            rec[kStatHdr + tid] = ((s_A[0][tid] + s_A[1][tid]) + (s_A[2][tid] + s_A[3][tid])) +
                                  (double)mc * ((s_redd[0] + s_redd[1]) + (s_redd[2] + s_redd[3]));
    } else if (drafts && tid < n) {
        rec[kStatHdr + tid] = (s_A[0][tid] + s_A[1][tid]) + (s_A[2][tid] + s_A[3][tid]);
    }
}

// =====================================================================================================
// Second-pass distances: total variation, and the two-draft grid policy's candidate mixtures.
// |p - q| (and log of a mixture) cannot be accumulated before the target row's normaliser is known, so
// these modes take one more pass over the rows: grid (chunk, position i < gamma, sequence b); every
// workgroup first combines the row's records from k_stats (lse_p), then sums, over its 4096-wide chunk,
//   MODE 0: |p - q_j|                         per draft j                (TVD, DW = n)
//   MODE 1: p (log p - log mix_c)             per candidate c = 0..10    (KL of the mixtures, n = 2)
//   MODE 2: |p - mix_c|                       per candidate c            (TVD of the mixtures, n = 2)
//   MODE 3: arg-max_v q_j(v)                  per draft j                (hard labels; needs no target row)
//   MODE 4: arg-max_v mix_c(v)                per candidate c            (hard labels, n = 2)
// with mix_c = (1 - c/10) q_1 + (c/10) q_2.  Chunk sums go to dist[b][i][c][chunk][0] (k_finish adds them);
// chunk arg-maxes go to dist[b][i][c][chunk][0..1] as ((value, runner-up value) as two floats, index), lowest
// index on ties.
// =====================================================================================================
struct DistArgs {
    int V, n, B, gamma, C3, RS, DW, Cd;
    const float* target;
    const float* dlogits;
    const double* dlse;
    const float* temperature;
    const double* stats;
    double* dist;
};

template <bool VEC, int MODE>
__global__ __launch_bounds__(kBlock) void k_dist(DistArgs a) {
    const int c = blockIdx.x, i = blockIdx.y, b = blockIdx.z, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = a.V, n = a.n, gamma = a.gamma;
    constexpr int NC = TABED_GRID_CANDIDATES;
    __shared__ double s_lse;
    __shared__ float s_hi[TABED_MAX_N], s_oml[TABED_MAX_N];
    __shared__ double s_sum[kWavesPerBlock][TABED_MAX_N];
    __shared__ ArgMax s_amx[kWavesPerBlock][TABED_MAX_N];
    __shared__ float s_sec[kWavesPerBlock][TABED_MAX_N];      // runner-up value beside every arg-max (mixtures only)

    const float* trow = a.target + ((size_t)b * (gamma + 1) + i) * V;
    const float* qbase = a.dlogits + (((size_t)i * a.B + b) * n) * V;
    const int cb = c * kChunkV;
    if (MODE >= 3) {
        // ---- hard labels: arg-max of every candidate distribution over this chunk
        const float T3 = a.temperature[b];
        const float invT3 = (T3 > 0.f) ? 1.f / T3 : 1.f;
        if (MODE == 3) {
            for (int j = 0; j < n; ++j) {                  // softmax is monotone: the arg-max of the raw logits
                ArgMax am{-INFINITY, 0x7fffffff};
                float4 y[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) y[u] = load4<VEC>(qbase + (size_t)j * V, cb + (u * kBlock + tid) * 4, V);
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = cb + (u * kBlock + tid) * 4 + e;
                        if (v < V) am = argmax_merge(am, ArgMax{f4get(y[u], e), v});
                    }
                am = wave_argmax(am);
                // fp32 logits compare exactly on both sides of any check: no runner-up is needed for these
                if (lane == 0) { s_amx[wave][j] = am; s_sec[wave][j] = -INFINITY; }
            }
        } else {
            if (tid < 2) {
                const double l = a.dlse[((size_t)i * a.B + b) * n + tid];
                const float hi = (float)l;
                s_hi[tid] = hi;
                s_oml[tid] = (float)(1.0 - (l - (double)hi));
            }
            float4 y0[4], y1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                y0[u] = load4<VEC>(qbase, cb + (u * kBlock + tid) * 4, V);
                y1[u] = load4<VEC>(qbase + (size_t)V, cb + (u * kBlock + tid) * 4, V);
            }
            __syncthreads();
            float q0[16], q1[16];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a0 = f4get(y0[u], e), a1 = f4get(y1[u], e);
                    q0[u * 4 + e] = (a0 > -INFINITY) ? __expf(a0 * invT3 - s_hi[0]) * s_oml[0] : 0.f;
                    q1[u * 4 + e] = (a1 > -INFINITY) ? __expf(a1 * invT3 - s_hi[1]) * s_oml[1] : 0.f;
                }
            for (int k = 0; k < NC; ++k) {
                const float w1 = (float)k / (float)(NC - 1), w0 = 1.f - w1;
                // the mixture is evaluated in fp32 here and in fp64 by a checker: the runner-up travels with the
                // arg-max so that a near-tie can be flagged where the label is known
                ArgMax am{-INFINITY, 0x7fffffff};
                float sec = -INFINITY;
#pragma unroll
                for (int x = 0; x < 16; ++x) {
                    const int v = cb + ((x >> 2) * kBlock + tid) * 4 + (x & 3);
                    if (v < V) {
                        const ArgMax cand{w0 * q0[x] + w1 * q1[x], v};
                        const ArgMax win = argmax_merge(am, cand);
                        sec = fmaxf(sec, win.i == cand.i ? am.v : cand.v);      // the loser's value
                        am = win;
                    }
                }
                const ArgMax wam = wave_argmax(am);
                const float wsec = wave_max((am.i == wam.i) ? sec : am.v);
                if (lane == 0) { s_amx[wave][k] = wam; s_sec[wave][k] = wsec; }
            }
        }
        __syncthreads();
        if (tid < a.DW) {
            ArgMax t = s_amx[0][tid];
            float sec = s_sec[0][tid];
            for (int w = 1; w < kWavesPerBlock; ++w) {
                const ArgMax o = s_amx[w][tid];
                const ArgMax win = argmax_merge(t, o);
                sec = fmaxf(fmaxf(sec, s_sec[w][tid]), (win.i == o.i && o.i != t.i) ? t.v : o.v);
                t = win;
            }
            double* rec = a.dist + ((((size_t)b * gamma + i) * a.DW + tid) * a.Cd + c) * 2;
            rec[0] = __builtin_bit_cast(double, make_float2(t.v, sec));       // (arg-max value, runner-up value)
            rec[1] = (double)t.i;
        }
        return;
    }
    float4 tx[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) tx[u] = load4<VEC>(trow, cb + (u * kBlock + tid) * 4, V);
    float4 yq[2][4];                                   // grid modes: both draft rows, requested up front
    if (MODE != 0) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int u = 0; u < 4; ++u) yq[j][u] = load4<VEC>(qbase + (size_t)j * V, cb + (u * kBlock + tid) * 4, V);
    }
    const float T = a.temperature[b];
    const float invT = (T > 0.f) ? 1.f / T : 1.f;
    if (tid < n) {
        const double l = a.dlse[((size_t)i * a.B + b) * n + tid];
        const float hi = (float)l;
        s_hi[tid] = hi;
        s_oml[tid] = (float)(1.0 - (l - (double)hi));
    }
    if (wave == 0) {                                   // lse of target row (b, i) from its records
        const double* r0 = a.stats + ((size_t)b * (gamma + 1) + i) * a.C3 * a.RS;
        double m = -INFINITY;
        for (int cc = lane; cc < a.C3; cc += kWave) m = fmax(m, r0[(size_t)cc * a.RS]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m = fmax(m, __shfl_xor(m, o));
        double Z = 0.0;
        for (int cc = lane; cc < a.C3; cc += kWave) {
            const double* r = r0 + (size_t)cc * a.RS;
            if (r[0] > -INFINITY) Z += r[1] * exp(r[0] - m);
        }
        Z = wave_sum(Z);
        if (lane == 0) s_lse = m + log(Z);
    }
    __syncthreads();
    const double lse = s_lse;
    const float lhi = (float)lse, loml = (float)(1.0 - (lse - (double)lhi));

    float pv[16], lp[16];                              // p and log p of this thread's 16 elements
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float xe = f4get(tx[u], e);
            const float st = xe * invT;
            const bool ok = xe > -INFINITY;
            pv[u * 4 + e] = ok ? __expf(st - lhi) * loml : 0.f;
            lp[u * 4 + e] = ok ? (st - lhi) + (loml - 1.f) : 0.f;
        }

    if (MODE == 0) {
        for (int j = 0; j < n; ++j) {
            float acc = 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float4 y = load4<VEC>(qbase + (size_t)j * V, cb + (u * kBlock + tid) * 4, V);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float ye = f4get(y, e);
                    const float q = (ye > -INFINITY) ? __expf(ye * invT - s_hi[j]) * s_oml[j] : 0.f;
                    acc += fabsf(pv[u * 4 + e] - q);
                }
            }
            const double t = wave_sum((double)acc);
            if (lane == 0) s_sum[wave][j] = t;
        }
    } else {
        // both drafts' probabilities of this thread's 16 elements, then one candidate mixture at a time
        float q0[16], q1[16];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a0 = f4get(yq[0][u], e), a1 = f4get(yq[1][u], e);
                q0[u * 4 + e] = (a0 > -INFINITY) ? __expf(a0 * invT - s_hi[0]) * s_oml[0] : 0.f;
                q1[u * 4 + e] = (a1 > -INFINITY) ? __expf(a1 * invT - s_hi[1]) * s_oml[1] : 0.f;
            }
        for (int k = 0; k < NC; ++k) {
            const float w1 = (float)k / (float)(NC - 1), w0 = 1.f - w1;
            float acc = 0.f;
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const float mix = w0 * q0[x] + w1 * q1[x];
                // bare v_log_f32 (log2): its ~1e-7 relative error is random per element and averages out under
                // sum p (..); a mixture below the normal range only occurs where p is negligible too
                if (MODE == 1) acc += (pv[x] > 0.f) ? pv[x] * (lp[x] * 1.44269504f - __builtin_amdgcn_logf(fmaxf(mix, 1e-37f))) : 0.f;
                else acc += fabsf(pv[x] - mix);
            }
            if (MODE == 1) acc *= 0.693147181f;            // back from log2 to natural log
            const double t = wave_sum((double)acc);
            if (lane == 0) s_sum[wave][k] = t;
        }
    }
    __syncthreads();
    if (tid < a.DW)
        a.dist[((((size_t)b * gamma + i) * a.DW + tid) * a.Cd + c) * 2] =
            (s_sum[0][tid] + s_sum[1][tid]) + (s_sum[2][tid] + s_sum[3][tid]);
}

static int pick_stats_unroll(const tabed_cfg& c, int nmax_u) {
    // Largest chunk that still gives the chip a few workgroups per compute unit.
    const long rows = (long)c.B * (c.gamma + 1);
    for (int U : {4, 2}) {
        if (U > nmax_u) continue;
        const long chunks = (c.V + kBlock * 4 * U - 1) / (kBlock * 4 * U);
        if (rows * chunks >= 1024) return U;           // measured on the serving shape: 1536 workgroups beat 768
    }
    return 1;
}

template <bool VEC, int N>
static void launch_stats_n(const ProfScope* prof, int U, dim3 grid, hipStream_t s, const StatsArgs& a) {
    if (U == 4) {
        if constexpr (N <= 4) launch(prof, k_stats<VEC, 4, N>, grid, dim3(kBlock), 0, s, a);
    } else if (U == 2) {
        launch(prof, k_stats<VEC, 2, N>, grid, dim3(kBlock), 0, s, a);
    } else {
        launch(prof, k_stats<VEC, 1, N>, grid, dim3(kBlock), 0, s, a);
    }
}

// =====================================================================================================
// Accept chain, distances, corrected / bonus token.
// Grid (chunk + 1, sequence b).  Every workgroup of a sequence first combines the chunk records of all
// gamma+1 target rows (fp64, chunk order), evaluates the gamma accept tests of Sec. 3 item 3 in parallel
// and takes k = the first failing position.  The last workgroup of the row (the "book-keeping" one) has
// no vocabulary chunk: it writes KL(p_i || q_i^(j)) and the bookkeeping outputs and, when asked to,
// advances the window and computes the next weights while its siblings work on the residual row.  For a sampling row the emitted token comes from f = max(0, p_k - q_k) (k < gamma)
// or f = p_gamma (k = gamma): every wave writes the mass of f over its 256-wide segments; the last
// workgroup of the sequence to arrive prefixes the segment masses in order, finds the segment the uniform
// falls into, and one wave re-evaluates that segment element by element.  A greedy row emits the arg-max of
// target row k and needs no vocabulary pass.
// =====================================================================================================
struct FinishArgs {
    int V, n, B, gamma, C3, RS, NSEG, C5;
    uint64_t seed, round;
    const float* target;
    const float* dlogits;
    const double* dlse;
    const int32_t* dtok;
    const float* dq;
    const float* weights;
    const float* temperature;
    const float* u_acc;
    const float* u_res;
    const double* stats;
    const double* dist;   // [B][gamma][DW][Cd] second-pass chunk sums, or nullptr (KL from the records)
    int DW, Cd;
    float dist_scale;     // 0.5 for total variation, 1 for KL
    int hard;             // 1: dist holds chunk arg-maxes and the distance is the token-mismatch indicator
    int hard_margin;      // 1: those arg-maxes are of fp32 mixtures: a near-tie flags the position
    int grid_kl;          // 1: the records of k_stats hold the KL sums of the DW candidate mixtures (no second pass)
    int fuse;             // 1: the call also advances every sequence's window and writes the next weights
    WindowArgs win;
    double* tstate;       // token tree: [B][kTsSlots] record of every sequence's walk, or nullptr (chain)
    float* wstage;        // [B][n] next weights, staged until every workgroup of the sequence has arrived
    double* seg;          // [B][2][NSEG]
    uint32_t* tickets;
    int32_t* accept_len;
    int32_t* out_tokens;
    float* dev;
    int32_t* n_valid;
    uint8_t* flags;
};

// exp(x - (hi + lo)), lo << 1.  The residual pass only locates a CDF crossing, whose margin (1e-6 of the
// total mass, flagged) is far above the ~1e-7 |x - hi| relative error of the fast exponential.
__device__ __forceinline__ float exp_shifted(float x, float hi, float one_minus_lo) {
    return __expf(x - hi) * one_minus_lo;
}

struct ResidRow {
    const float* trow;
    const float* qrows;   // n rows, stride V
    float invT, pmax, pinvZ;
    bool bonus;
};

// f and p for S groups of four consecutive elements starting at v[s] (v[s] % 4 == 0; a group at or past V
// contributes zeros).  Every load is issued before the first use; N is the compile-time number of drafts
// (0 = run time, one batch of S loads per draft).
template <bool VEC, int N, int S>
__device__ __forceinline__ void resid_eval(const ResidRow& r, int n, int V, const int (&v)[S], const float* s_hi,
                                           const float* s_lo, const float* s_w, float (&f)[S][4], float (&p)[S][4],
                                           float (&q)[S][4]) {
    float4 tx[S];
#pragma unroll
    for (int s = 0; s < S; ++s) tx[s] = load4<VEC>(r.trow, v[s], V);
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int e = 0; e < 4; ++e) q[s][e] = 0.f;
    if (!r.bonus) {
        if (N > 0) {
            float4 dx[(N > 0) ? N : 1][S];
#pragma unroll
            for (int j = 0; j < N; ++j)
#pragma unroll
                for (int s = 0; s < S; ++s) dx[j][s] = load4<VEC>(r.qrows + (size_t)j * V, v[s], V);
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const float w = s_w[j], hi = s_hi[j], lo = s_lo[j];
#pragma unroll
                for (int s = 0; s < S; ++s)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float ye = f4get(dx[j][s], e);
                        if (ye > -INFINITY) q[s][e] += w * exp_shifted(ye * r.invT, hi, lo);
                    }
            }
        } else {
            for (int j = 0; j < n; ++j) {
                float4 y[S];
#pragma unroll
                for (int s = 0; s < S; ++s) y[s] = load4<VEC>(r.qrows + (size_t)j * V, v[s], V);
                const float w = s_w[j], hi = s_hi[j], lo = s_lo[j];
#pragma unroll
                for (int s = 0; s < S; ++s)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float ye = f4get(y[s], e);
                        if (ye > -INFINITY) q[s][e] += w * exp_shifted(ye * r.invT, hi, lo);
                    }
            }
        }
    }
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float xe = f4get(tx[s], e);
            const float pe = (xe > -INFINITY) ? __expf(xe * r.invT - r.pmax) * r.pinvZ : 0.f;
            p[s][e] = pe;
            f[s][e] = r.bonus ? pe : fmaxf(0.f, pe - q[s][e]);
        }
}

// Arg-max over the chunk arg-maxes of one (position, candidate): records are ((value, runner-up), index).
// *near: the runner-up over the whole row is within the margin of the winner.
__device__ __forceinline__ int hard_pred(const double* rec, int Cd, bool* near) {
    ArgMax am{-INFINITY, 0x7fffffff};
    float sec = -INFINITY;
    for (int cc = 0; cc < Cd; ++cc) {
        const float2 vs = __builtin_bit_cast(float2, rec[cc * 2]);
        const ArgMax o{vs.x, (int)rec[cc * 2 + 1]};
        const ArgMax win = argmax_merge(am, o);
        sec = fmaxf(fmaxf(sec, vs.y), (win.i == o.i && o.i != am.i) ? am.v : o.v);
        am = win;
    }
    *near = (am.v - sec) < kMargin * fabsf(am.v);
    return am.i;
}

template <bool VEC, int N>
__global__ __launch_bounds__(kBlock) void k_finish(FinishArgs a) {
    extern __shared__ __attribute__((aligned(16))) double s_scale[];   // [gamma+1][C3]: exp(m_c - m_row)
    const int c = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = a.V, n = (N > 0) ? N : a.n, gamma = a.gamma, NSEG = a.NSEG, C3 = a.C3, RS = a.RS;

    __shared__ double s_rowm[TABED_MAX_GAMMA + 1], s_rowZ[TABED_MAX_GAMMA + 1], s_rowlse[TABED_MAX_GAMMA + 1];
    __shared__ int s_rowam[TABED_MAX_GAMMA + 1];
    __shared__ int s_ok[TABED_MAX_GAMMA];
    __shared__ uint32_t s_aflag[TABED_MAX_GAMMA + 1];
    __shared__ float s_hi[TABED_MAX_GAMMA][TABED_MAX_N], s_lo[TABED_MAX_GAMMA][TABED_MAX_N], s_w[TABED_MAX_N];
    __shared__ double s_redd[kWavesPerBlock];
    __shared__ int s_last, s_first[kWavesPerBlock], s_lastw[kWavesPerBlock], s_seg;
    __shared__ double s_prefix;
    __shared__ double s_wpart[64], s_wx[TABED_MAX_N];    // fused window update (one wave)
    __shared__ int s_y[TABED_MAX_GAMMA];                 // drafted tokens (hard labels)

    // ---- everything that does not depend on another load is requested first
    int y = -1;
    float rawy = 0.f, uacc = 0.f, qy = 0.f;
    if (tid < gamma) {
        y = a.dtok[(size_t)b * gamma + tid];
        uacc = a.u_acc ? a.u_acc[(size_t)b * gamma + tid] : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)tid, 1);
        qy = a.dq[(size_t)b * gamma + tid];
        s_y[tid] = y;
    }
    for (int q = tid; q < gamma * n; q += kBlock) {      // draft log-sum-exps of every position, split hi + lo
        const double l = a.dlse[((size_t)(q / n) * a.B + b) * n + (q % n)];
        const float hi = (float)l;
        s_hi[q / n][q % n] = hi;
        s_lo[q / n][q % n] = (float)(1.0 - (l - (double)hi));      // 1 - lo, the first-order factor of exp(-lo)
    }
    if (tid < n) s_w[tid] = a.weights[(size_t)b * n + tid];
    const float T = a.temperature[b];

    // ---- combine the chunk records of every target row.  A row's C3 chunks sit in an aligned group of
    //      C3p lanes (C3p = power of two >= C3), so one wave combines 64 / C3p rows per pass with one
    //      load round trip; rows with more than 64 chunks fall back to one wave per row.
    const double* sb = a.stats + (size_t)b * (gamma + 1) * C3 * RS;
    if (C3 <= kWave) {
        int C3p = 1;
        while (C3p < C3) C3p <<= 1;
        const int rows_per_pass = kWave / C3p;
        const int cc = lane & (C3p - 1);
        for (int row0 = wave * rows_per_pass; row0 <= gamma; row0 += kWavesPerBlock * rows_per_pass) {
            const int row = row0 + lane / C3p;
            const bool live = (row <= gamma && cc < C3);
            double r0v = -INFINITY, r1v = 0.0;
            ArgMax am{-INFINITY, 0x7fffffff};
            if (live) {
                const double* r = sb + ((size_t)row * C3 + cc) * RS;
                r0v = r[0]; r1v = r[1];
                am = ArgMax{(float)r[2], (int)r[3]};
            }
            // all-reduce inside aligned groups of C3p lanes: DPP for the first four doublings (no LDS traffic),
            // ds_bpermute only beyond a 16-lane row
            double m = r0v;
            if (C3p > 1) m = fmax(m, dpp_f64<kDppXor1>(m));
            if (C3p > 2) m = fmax(m, dpp_f64<kDppXor2>(m));
            if (C3p > 4) m = fmax(m, dpp_f64<kDppHalfMirror>(m));
            if (C3p > 8) m = fmax(m, dpp_f64<kDppMirror>(m));
            for (int o = 16; o < C3p; o <<= 1) m = fmax(m, __shfl_xor(m, o));
            const double sc = (r0v > -INFINITY) ? exp(r0v - m) : 0.0;
            if (live) s_scale[row * C3 + cc] = sc;
            double Z = r1v * sc;
            if (C3p > 1) { Z += dpp_f64<kDppXor1>(Z); am = argmax_dpp_step<kDppXor1>(am); }
            if (C3p > 2) { Z += dpp_f64<kDppXor2>(Z); am = argmax_dpp_step<kDppXor2>(am); }
            if (C3p > 4) { Z += dpp_f64<kDppHalfMirror>(Z); am = argmax_dpp_step<kDppHalfMirror>(am); }
            if (C3p > 8) { Z += dpp_f64<kDppMirror>(Z); am = argmax_dpp_step<kDppMirror>(am); }
            for (int o = 16; o < C3p; o <<= 1) {
                Z += __shfl_xor(Z, o);
                const ArgMax other{__shfl_xor(am.v, o), __shfl_xor(am.i, o)};
                am = argmax_merge(am, other);
            }
            if (live && cc == 0) { s_rowm[row] = m; s_rowZ[row] = Z; s_rowlse[row] = m + log(Z); s_rowam[row] = am.i; }
        }
    } else {
        for (int row = wave; row <= gamma; row += kWavesPerBlock) {
            const double* r0 = sb + (size_t)row * C3 * RS;
            double m = -INFINITY;
            for (int cc = lane; cc < C3; cc += kWave) m = fmax(m, r0[(size_t)cc * RS]);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) m = fmax(m, __shfl_xor(m, o));
            double Z = 0.0;
            ArgMax am{-INFINITY, 0x7fffffff};
            for (int cc = lane; cc < C3; cc += kWave) {
                const double* r = r0 + (size_t)cc * RS;
                const double sc = (r[0] > -INFINITY) ? exp(r[0] - m) : 0.0;
                s_scale[row * C3 + cc] = sc;
                Z += r[1] * sc;
                am = argmax_merge(am, ArgMax{(float)r[2], (int)r[3]});
            }
            Z = wave_sum(Z);
            am = wave_argmax(am);
            if (lane == 0) { s_rowm[row] = m; s_rowZ[row] = Z; s_rowlse[row] = m + log(Z); s_rowam[row] = am.i; }
        }
    }
    const bool greedy = !(T > 0.f);
    const bool book = (c == a.C5);                        // the book-keeping workgroup of this sequence
    if (greedy && !book) return;
    const float invT = greedy ? 1.f : 1.f / T;
    const bool y_ok = (y >= 0 && y < V);
    if (tid < gamma && y_ok && !greedy) rawy = a.target[((size_t)b * (gamma + 1) + tid) * V + y];
    __syncthreads();

    // ---- gamma accept tests in parallel, k = first failure
    if (tid < gamma) {
        uint32_t flag = 0;
        bool ok;
        if (!y_ok) { ok = false; flag |= TABED_FLAG_DEGENERATE; }
        else if (greedy) ok = (y == s_rowam[tid]);
        else {
            const float py = (float)exp((double)(rawy * invT) - s_rowlse[tid]);
            const float lhs = uacc * qy;
            ok = lhs < py;
            if (fabs((double)lhs - (double)py) < (double)kMargin * fmax((double)lhs, (double)py))
                flag |= TABED_FLAG_ACCEPT_MARGIN;
        }
        s_ok[tid] = ok ? 1 : 0;
        s_aflag[tid] = flag;
    }
    if (tid == gamma) s_aflag[gamma] = 0;
    __syncthreads();
    int k = 0;
    while (k < gamma && s_ok[k]) ++k;
    const size_t out_idx = (size_t)b * (gamma + 1) + k;

    // ---- this workgroup's share of the residual (or bonus) row: 2 segments per wave, loads first
    ResidRow r;
    r.bonus = (k == gamma);
    r.invT = invT;
    r.trow = a.target + out_idx * V;
    r.pmax = (float)s_rowm[k];
    r.pinvZ = (float)(1.0 / s_rowZ[k]);
    r.qrows = r.bonus ? a.dlogits : a.dlogits + ((size_t)k * a.B + b) * n * V;
    const float* hi_k = s_hi[r.bonus ? 0 : k];
    const float* lo_k = s_lo[r.bonus ? 0 : k];
    constexpr int kSegPerChunk = kResidChunkV / kSegV;            // 8
    constexpr int kSegPerWave = kSegPerChunk / kWavesPerBlock;    // 2
    float f[kSegPerWave][4], p[kSegPerWave][4], qmix[kSegPerWave][4];
    int vs[kSegPerWave];
    if (!greedy && !book) {
#pragma unroll
        for (int s = 0; s < kSegPerWave; ++s) vs[s] = (c * kSegPerChunk + wave + s * kWavesPerBlock) * kSegV + lane * 4;
        resid_eval<VEC, N, kSegPerWave>(r, n, V, vs, hi_k, lo_k, s_w, f, p, qmix);
    }

    if (book) {
        if (a.dist == nullptr) {
            // ---- distances: thread per (position, draft or candidate mixture), chunks in order with the scales
            //      computed above.  KL(p || q_j) = A_j / Z - lse_p + lse_j; a mixture's sums already hold its logarithm.
            const int dw = a.grid_kl ? a.DW : n;
            for (int q = tid; q < gamma * dw; q += kBlock) {
                const int ii = q / dw, j = q % dw;
                const double* r0 = sb + (size_t)ii * C3 * RS + kStatHdr + j;
                double A = 0.0;
#pragma unroll 8
                for (int cc = 0; cc < C3; ++cc) A += r0[(size_t)cc * RS] * s_scale[ii * C3 + cc];
                const double kl = A / s_rowZ[ii] - s_rowlse[ii] + (a.grid_kl ? 0.0 : a.dlse[((size_t)ii * a.B + b) * n + j]);
                publish_store(&a.dev[((size_t)b * gamma + ii) * dw + j], (float)kl);
            }
        } else if (!a.hard) {
            // ---- distances from the second pass: add the chunk sums in chunk order
            for (int q = tid; q < gamma * a.DW; q += kBlock) {
                const double* r0 = a.dist + ((size_t)b * gamma * a.DW + q) * a.Cd * 2;
                double D = 0.0;
                for (int cc = 0; cc < a.Cd; ++cc) D += r0[cc * 2];
                publish_store(&a.dev[(size_t)b * gamma * a.DW + q], (float)((double)a.dist_scale * D));
            }
        } else {
            // ---- hard labels: 1 where a candidate's arg-max differs from the token emitted at the position.
            //      The label of the rejected position of a sampling row is the corrected token, which only
            //      the sampler's last workgroup knows: that entry is written there.
            for (int q = tid; q < gamma * a.DW; q += kBlock) {
                const int ii = q / a.DW;
                if (ii == k && !greedy) continue;
                const int label = ii < k ? s_y[ii] : (ii == k ? s_rowam[k] : -1);
                bool near;
                const int pred = hard_pred(a.dist + ((size_t)b * gamma * a.DW + q) * a.Cd * 2, a.Cd, &near);
                publish_store(&a.dev[(size_t)b * gamma * a.DW + q], pred == label ? 0.f : 1.f);
                if (near && a.hard_margin && ii <= k) atomicOr(&s_aflag[ii], (uint32_t)TABED_FLAG_SAMPLE_MARGIN);
            }
            __syncthreads();                               // (uniform: book and a.hard are) the flags are complete
        }
        if (tid <= gamma) {
            // accepted prefix, -1 padding, flags of the tests that were evaluated; slot k belongs to the sampler
            if (tid != k) {
                a.out_tokens[(size_t)b * (gamma + 1) + tid] = tid < k ? y : -1;
                a.flags[(size_t)b * (gamma + 1) + tid] = (uint8_t)(tid < k ? s_aflag[tid] : 0u);
            } else if (greedy) {
                a.out_tokens[out_idx] = s_rowam[k];
                a.flags[out_idx] = (uint8_t)s_aflag[k];
            }
        }
        if (tid == 0) {
            a.accept_len[b] = k;
            a.n_valid[b] = k + 1 < gamma ? k + 1 : gamma;
            if (a.tstate != nullptr && greedy) {           // token tree: where the trunk stopped and what the target wants there
                double* ts = a.tstate + (size_t)b * kTsSlots;
                ts[kTsK] = (double)k;
                ts[kTsArgmax] = (double)s_rowam[k];
                ts[kTsZ1] = 0.0;
            }
        }
    }
    const int nv_k = k + 1 < gamma ? k + 1 : gamma;
    if (greedy) {
        // a greedy row is complete here: its single workgroup also advances the window when asked to
        if (a.fuse) {
            publish_barrier();                             // the distances above are acknowledged
            if (tid < kWave) window_update<true>(a.win, b, lane, a.dev, nv_k, s_wpart, s_wx);
        }
        return;
    }

    double* segR = a.seg + ((size_t)b * 2 + 0) * NSEG;
    double* segP = a.seg + ((size_t)b * 2 + 1) * NSEG;
    if (book) {
        // window + next weights, off the critical path of the sampler.  The weights are staged: the buffer
        // they go to may be the one the siblings are still reading this block's weights from.
        if (a.fuse && !a.hard) {
            publish_barrier();                             // the distances above are acknowledged
            if (tid < kWave) {
                WindowArgs wa = a.win;
                wa.weights = a.wstage;
                window_update<true>(wa, b, lane, a.dev, nv_k, s_wpart, s_wx);
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < kSegPerWave; ++s) {
            const int seg = c * kSegPerChunk + wave + s * kWavesPerBlock;
            const double mf = (double)wave_sum((f[s][0] + f[s][1]) + (f[s][2] + f[s][3]));
            const double mp = (double)wave_sum((p[s][0] + p[s][1]) + (p[s][2] + p[s][3]));
            if (lane == 0 && seg < NSEG) { publish_store(&segR[seg], mf); publish_store(&segP[seg], mp); }
        }
    }
    publish_barrier();                                     // every wave's published stores are acknowledged
    if (tid == 0) s_last = arrive(&a.tickets[b], (uint32_t)(a.C5 + 1)) ? 1 : 0;
    __syncthreads();
    if (!s_last) return;
    if (a.fuse && !a.hard && tid < n) a.win.weights[(size_t)b * n + tid] = published_load(&a.wstage[(size_t)b * n + tid]);
    // hard labels: the rejected position's distances and the window update wait for the corrected token
    // returns the flag bit of a near-tie among the mixtures' arg-maxes at position k
    auto finish_hard = [&](int tok) -> uint32_t {          // wave 0 only
        bool any = false;
        if (k < gamma)
            for (int cidx = lane; cidx < a.DW; cidx += kWave) {
                bool near;
                const int pred = hard_pred(a.dist + (((size_t)b * gamma + k) * a.DW + cidx) * a.Cd * 2, a.Cd, &near);
                publish_store(&a.dev[((size_t)b * gamma + k) * a.DW + cidx], pred == tok ? 0.f : 1.f);
                any = any || near;
            }
        const uint32_t extra = (a.hard_margin && __ballot(any)) ? (uint32_t)TABED_FLAG_SAMPLE_MARGIN : 0u;
        if (a.fuse) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's published distances are acknowledged
            window_update<true>(a.win, b, lane, a.dev, nv_k, s_wpart, s_wx);
        }
        return extra;
    };

    // ---- last workgroup of sequence b: locate the segment, then the token
    const int S = (NSEG + kBlock - 1) / kBlock;
    const int g0 = min(NSEG, tid * S), g1 = min(NSEG, g0 + S);
    uint32_t flag = s_aflag[k];
    double runR = 0.0, runP = 0.0;
    for (int g = g0; g < g1; ++g) { runR += published_load(&segR[g]); runP += published_load(&segP[g]); }
    double run = runP;
    const double* mass = segP;
    double Z1 = 0.0;
    if (!r.bonus) {
        const double Zr = block_sum(runR, s_redd);
        if (Zr > 0.0) { run = runR; mass = segR; Z1 = Zr; }
        else { r.bonus = true; flag |= TABED_FLAG_DEGENERATE; }   // empty residual: draw from p_k
    }
    if (a.tstate != nullptr && tid == 0) {                 // token tree: the first residual level is known here
        double* ts = a.tstate + (size_t)b * kTsSlots;
        ts[kTsK] = (double)k;
        ts[kTsRowMax] = s_rowm[k];
        ts[kTsRowZ] = s_rowZ[k];
        ts[kTsZ1] = Z1;                                    // 0: all gamma accepted, or an empty residual
        ts[kTsArgmax] = (double)s_rowam[k];
    }
    double Z;
    const double excl = block_exclusive_scan(run, s_redd, &Z);
    const float u = a.u_res ? a.u_res[b] : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)gamma, 0);
    const double target = (double)u * Z;
    const int owner = block_find_owner(excl, run, target, s_first, s_lastw);
    if (owner < 0) {
        if (tid == 0) {
            a.out_tokens[out_idx] = 0;
            a.flags[out_idx] = (uint8_t)(flag | TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE);
        }
        if (a.hard && tid < kWave) finish_hard(0);
        return;
    }
    if (tid == owner) {
        double P = excl, Plast = excl;
        int gstar = -1, glast = g0;
        for (int g = g0; g < g1; ++g) {
            const double mg = published_load(&mass[g]);
            if (mg > 0.0) { glast = g; Plast = P; }
            if (P + mg > target) { gstar = g; break; }
            P += mg;
        }
        if (gstar < 0) { gstar = glast; P = Plast; }
        s_seg = gstar;
        s_prefix = P;
    }
    __syncthreads();
    if (tid >= kWave) return;
    const int v1[1] = {s_seg * kSegV + lane * 4};
    float f1[1][4], p1[1][4], q1[1][4];
    resid_eval<VEC, N, 1>(r, n, V, v1, hi_k, lo_k, s_w, f1, p1, q1);
    const int v = v1[0];
    const double l1 = (double)f1[0][0], l2 = l1 + (double)f1[0][1], l3 = l2 + (double)f1[0][2], l4 = l3 + (double)f1[0][3];
    const double base = s_prefix + (wave_inclusive_scan(l4) - l4);
    const double cdf[4] = {base + l1, base + l2, base + l3, base + l4};
    int hit = -1, lastlive = -1;
#pragma unroll
    for (int e = 3; e >= 0; --e) {
        if (f1[0][e] > 0.f && cdf[e] > target) hit = e;
        if (lastlive < 0 && f1[0][e] > 0.f) lastlive = e;
    }
    const unsigned long long cross = __ballot(hit >= 0);
    const unsigned long long live = __ballot(lastlive >= 0);
    int pick;
    if (cross) pick = __ffsll((long long)cross) - 1;
    else if (live) { pick = 63 - __clzll((long long)live); flag |= TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE; }
    else { pick = 0; flag |= TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE; }
    if (a.hard) {
        const int e = cross ? hit : (live ? lastlive : 0);
        const int mine = (v + e < V) ? v + e : V - 1;
        flag |= finish_hard(__builtin_amdgcn_readlane(mine, pick));
    }
    if (lane == pick) {
        const int e = cross ? hit : (live ? lastlive : 0);
        const int tok = v + e;
        const double tol = (double)kMargin * Z;
        const double fe = (double)(e == 0 ? f1[0][0] : e == 1 ? f1[0][1] : e == 2 ? f1[0][2] : f1[0][3]);
        const double hi_edge = e == 0 ? cdf[0] : e == 1 ? cdf[1] : e == 2 ? cdf[2] : cdf[3];
        if (fabs(hi_edge - target) < tol && tok + 1 < V) flag |= TABED_FLAG_SAMPLE_MARGIN;
        if (tok > 0 && fabs((hi_edge - fe) - target) < tol) flag |= TABED_FLAG_SAMPLE_MARGIN;
        a.out_tokens[out_idx] = tok < V ? tok : V - 1;
        a.flags[out_idx] = (uint8_t)flag;
    }
}

hipError_t launch_verify(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round,
                         const float* target_logits, const float* draft_logits, const double* draft_lse,
                         const int32_t* draft_tokens, const float* draft_q, const float* weights,
                         const float* temperature, const float* u_acc, const float* u_res, int32_t* accept_len,
                         int32_t* out_tokens, float* dev, int32_t* n_valid, uint8_t* flags, float* ring,
                         int32_t* ring_head, int32_t* ring_count, float* next_weights, bool tree, hipStream_t s) {
    const bool vec = (c.V % 4 == 0);
    // the KL of the two-draft grid's mixtures rides in the statistics pass (vectorised rows only)
    const bool grid_in_stats = (c.policy == 2 && c.distance == 0 && vec);
    const bool second_pass = (c.distance != 0 || (c.policy == 2 && !grid_in_stats));   // distances that take a pass of their own
    const int ncomp = (vec && (c.n == 2 || c.n == 4 || c.n == 8)) ? c.n : 0;   // compile-time draft counts
    const int U = pick_stats_unroll(c, ncomp == 8 ? 2 : 4);
    const int C3 = (c.V + kBlock * 4 * U - 1) / (kBlock * 4 * U);
    {
        ProfScope prof(TABED_K_STATS, s);
        StatsArgs a;
        a.V = c.V; a.n = c.n; a.B = c.B; a.gamma = c.gamma; a.RS = L.RS; a.C3 = C3;
        a.with_drafts = second_pass ? 0 : 1;
        a.grid = grid_in_stats ? 1 : 0;
        a.target = target_logits; a.dlogits = draft_logits; a.dlse = draft_lse; a.temperature = temperature;
        a.stats = reinterpret_cast<double*>(ws + L.off_stats);
        const dim3 grid(C3, c.gamma + 1, c.B);
        if (!vec) launch_stats_n<false, 0>(&prof, U, grid, s, a);
        else if (ncomp == 2) launch_stats_n<true, 2>(&prof, U, grid, s, a);
        else if (ncomp == 4) launch_stats_n<true, 4>(&prof, U, grid, s, a);
        else if (ncomp == 8) launch_stats_n<true, 8>(&prof, U, grid, s, a);
        else launch_stats_n<true, 0>(&prof, U, grid, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (second_pass) {
            ProfScope dprof(TABED_K_DIST, s);              // a dispatch of its own: its own event pair
            DistArgs d;
            d.V = c.V; d.n = c.n; d.B = c.B; d.gamma = c.gamma; d.C3 = C3; d.RS = L.RS; d.DW = L.DW; d.Cd = L.Cd;
            d.target = target_logits; d.dlogits = draft_logits; d.dlse = draft_lse; d.temperature = temperature;
            d.stats = a.stats;
            d.dist = reinterpret_cast<double*>(ws + L.off_dist);
            const dim3 gd(L.Cd, c.gamma, c.B);
            const int mode = (c.distance == 2) ? (c.policy != 2 ? 3 : 4) : (c.policy != 2) ? 0 : (c.distance == 0 ? 1 : 2);
            if (vec) {
                if (mode == 0) launch(&dprof, k_dist<true, 0>, gd, dim3(kBlock), 0, s, d);
                else if (mode == 1) launch(&dprof, k_dist<true, 1>, gd, dim3(kBlock), 0, s, d);
                else if (mode == 2) launch(&dprof, k_dist<true, 2>, gd, dim3(kBlock), 0, s, d);
                else if (mode == 3) launch(&dprof, k_dist<true, 3>, gd, dim3(kBlock), 0, s, d);
                else launch(&dprof, k_dist<true, 4>, gd, dim3(kBlock), 0, s, d);
            } else {
                if (mode == 0) launch(&dprof, k_dist<false, 0>, gd, dim3(kBlock), 0, s, d);
                else if (mode == 1) launch(&dprof, k_dist<false, 1>, gd, dim3(kBlock), 0, s, d);
                else if (mode == 2) launch(&dprof, k_dist<false, 2>, gd, dim3(kBlock), 0, s, d);
                else if (mode == 3) launch(&dprof, k_dist<false, 3>, gd, dim3(kBlock), 0, s, d);
                else launch(&dprof, k_dist<false, 4>, gd, dim3(kBlock), 0, s, d);
            }
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    ProfScope prof(TABED_K_RESID, s);
    FinishArgs a;
    a.V = c.V; a.n = c.n; a.B = c.B; a.gamma = c.gamma; a.C3 = C3; a.RS = L.RS; a.NSEG = L.NSEG; a.C5 = L.C5;
    a.seed = c.seed; a.round = round;
    a.target = target_logits; a.dlogits = draft_logits; a.dlse = draft_lse; a.dtok = draft_tokens; a.dq = draft_q;
    a.weights = weights; a.temperature = temperature; a.u_acc = u_acc; a.u_res = u_res;
    a.stats = reinterpret_cast<const double*>(ws + L.off_stats);
    a.dist = second_pass ? reinterpret_cast<const double*>(ws + L.off_dist) : nullptr;
    a.DW = L.DW; a.Cd = L.Cd; a.dist_scale = (c.distance == 1) ? 0.5f : 1.f; a.hard = (c.distance == 2) ? 1 : 0;
    a.hard_margin = (c.distance == 2 && c.policy == 2) ? 1 : 0;
    a.grid_kl = grid_in_stats ? 1 : 0;
    a.fuse = (ring != nullptr) ? 1 : 0;
    a.win = window_args(c, round + 1, ring, ring_head, ring_count, next_weights);   // the weights of the NEXT round
    a.wstage = reinterpret_cast<float*>(ws + L.off_wstage);
    a.tstate = tree ? reinterpret_cast<double*>(ws + L.off_tstate) : nullptr;
    a.seg = reinterpret_cast<double*>(ws + L.off_seg);
    a.tickets = reinterpret_cast<uint32_t*>(ws + L.off_tickets) + 2 * c.B;
    a.accept_len = accept_len; a.out_tokens = out_tokens; a.dev = dev; a.n_valid = n_valid; a.flags = flags;
    const dim3 grid(L.C5 + 1, c.B);                      // + the book-keeping workgroup of every sequence
    const size_t lds = sizeof(double) * (size_t)(c.gamma + 1) * C3;
    if (!vec) launch(&prof, k_finish<false, 0>, grid, dim3(kBlock), lds, s, a);
    else if (ncomp == 2) launch(&prof, k_finish<true, 2>, grid, dim3(kBlock), lds, s, a);
    else if (ncomp == 4) launch(&prof, k_finish<true, 4>, grid, dim3(kBlock), lds, s, a);
    else if (ncomp == 8) launch(&prof, k_finish<true, 8>, grid, dim3(kBlock), lds, s, a);
    else launch(&prof, k_finish<true, 0>, grid, dim3(kBlock), lds, s, a);
    return hipGetLastError();
}

// =====================================================================================================
// Token tree (Sec. 6.1, "Verification: Integrating Token Tree"): width sibling candidates per position, all
// from the position's ensembled distribution; candidate 0 is the trunk token the chain verifies, candidates
// 1..width-1 are leaves.  tabed_verify's kernels walk the trunk and leave, per sequence, where it stopped (k),
// the target row's normaliser there and the mass Z_1 of the first residual.  The passes below finish the walk
// at position k by multi-round rejection sampling: with f_0 = p_k, Z_0 = 1 and
//     f_c(v) = max(0, f_{c-1}(v) / Z_{c-1} - q_k(v)),   Z_c = sum_v f_c(v),
// sibling c is accepted iff u_c q_k(y_c) Z_c < f_c(y_c); an accepted sibling is emitted and followed by a
// bonus token from the target's distribution after it (its leaf row); if all are rejected the corrected
// token comes from f_width.  k_tree_begin decides sibling 1 (Z_1 is known), k_tree_level<L> computes level
// L >= 2 for the sequences still undecided and either decides sibling L or (L = width) draws the corrected
// token, k_tree_bonus draws the token after an accepted leaf.  Sequences whose walk is over skip every pass.
// =====================================================================================================
struct TreeArgs {
    int V, n, B, gamma, S, NSEG, C5;       // S = width - 1 siblings per position
    uint64_t seed, round;
    const float* target;                   // [B,gamma+1,V]
    const float* leaf_logits;              // [B,gamma,S,V]
    const float* dlogits;                  // [gamma,B,n,V]
    const double* dlse;                    // [gamma,B,n]
    const int32_t* sib_tokens;             // [B,gamma,S]
    const float* sib_q;                    // [B,gamma,S]
    const float* weights;
    const float* temperature;
    const float* u_res;
    const float* u_acc_sib;                // [B,gamma,S] or nullptr
    double* tstate;                        // [B][kTsSlots]
    const double* segP;                    // [B][2][NSEG] of tabed_verify's residual pass: slot 1 = masses of p_k
    double* tseg;                          // [B][2][NSEG]
    uint32_t* tickets;                     // [B] of this pass
    int32_t* out_tokens;
    uint8_t* flags;
    int32_t* leaf;
    int32_t* n_out;
};

// f_L(y) / Z_L's numerator chain at one token, in fp64, on the interface value q(y):
// returns f_{L-1}(y) / Z_{L-1} (the minuend of level L) given p(y), q(y) and the masses of the lower levels.
__device__ __forceinline__ double tree_minuend(int L, double py, double qy, double Z1, double Z2) {
    double m = py;                                          // level 1: f_0 / Z_0 = p
    if (L >= 2) m = fmax(0.0, m - qy) / Z1;
    if (L >= 3) m = fmax(0.0, m - qy) / Z2;
    return m;
}

// Sibling L's accept test (Z = Z_L).  Returns true if accepted; *flag gets the margin bit.
__device__ __forceinline__ bool tree_test(int L, double py, double qy, double Z1, double Z2, double Z, float u, uint32_t* flag) {
    const double minuend = tree_minuend(L, py, qy, Z1, Z2);
    const double fy = fmax(0.0, minuend - qy), lhs = (double)u * qy * Z;
    if (fabs(lhs - fy) < (double)kMargin * fmax(minuend, qy)) *flag |= TABED_FLAG_ACCEPT_MARGIN;
    return lhs < fy;
}

__global__ __launch_bounds__(64) void k_tree_begin(TreeArgs a) {
    const int b = blockIdx.x;
    if (threadIdx.x != 0) return;
    double* ts = a.tstate + (size_t)b * kTsSlots;
    const int gamma = a.gamma, S = a.S, V = a.V;
    const int k = (int)ts[kTsK];
    const float T = a.temperature[b];
    const bool greedy = !(T > 0.f);
    int status = kTreeDone, index = 0;
    a.leaf[b] = 0;
    a.n_out[b] = k + 1;
    if (k < gamma && S > 0) {
        const size_t so = ((size_t)b * gamma + k) * S;
        if (greedy) {
            const int top = (int)ts[kTsArgmax];
            for (int sidx = 1; sidx <= S && status == kTreeDone; ++sidx)
                if (a.sib_tokens[so + sidx - 1] == top) { status = kTreeLeaf; index = sidx; }
        } else if (ts[kTsZ1] > 0.0) {
            // the chain's corrected token (drawn from level 1) is replaced: by a leaf, or by a draw from level width
            uint32_t flag = a.flags[(size_t)b * (gamma + 1) + k] & ~(uint32_t)(TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE);
            const int y = a.sib_tokens[so];
            status = kTreePending; index = 2;
            if (y >= 0 && y < V) {
                const double lse = ts[kTsRowMax] + log(ts[kTsRowZ]);
                const double py = exp((double)(a.target[((size_t)b * (gamma + 1) + k) * V + y] * (1.f / T)) - lse);
                const float u = a.u_acc_sib ? a.u_acc_sib[so]
                                            : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)k + kSiblingStride, 1);
                if (tree_test(1, py, (double)a.sib_q[so], 0.0, 0.0, ts[kTsZ1], u, &flag)) { status = kTreeLeaf; index = 1; }
            } else {
                flag |= TABED_FLAG_DEGENERATE;
            }
            a.flags[(size_t)b * (gamma + 1) + k] = (uint8_t)flag;
        }
    }
    ts[kTsStatus] = (double)status;
    ts[kTsIndex] = (double)index;
}

// Locates, in the workgroup that finishes a sequence, the 256-wide segment whose prefix of masses crosses
// target = u * Z; thread `tid` owns segments [g0, g1).  Returns false if every mass is zero.
__device__ __forceinline__ bool tree_pick_segment(const double* mass, int g0, int g1, double excl, double run, double target,
                                                  int* s_first, int* s_lastw, int* s_seg, double* s_prefix) {
    const int owner = block_find_owner(excl, run, target, s_first, s_lastw);
    if (owner < 0) return false;
    if ((int)threadIdx.x == owner) {
        double P = excl, Plast = excl;
        int gstar = -1, glast = g0;
        for (int g = g0; g < g1; ++g) {
            const double mg = published_load(&mass[g]);
            if (mg > 0.0) { glast = g; Plast = P; }
            if (P + mg > target) { gstar = g; break; }
            P += mg;
        }
        if (gstar < 0) { gstar = glast; P = Plast; }
        *s_seg = gstar;
        *s_prefix = P;
    }
    __syncthreads();
    return true;
}

// One wave: given the four values of every lane's group inside the chosen segment, the token where the prefix
// crosses target, with the margin flags of the sampler.  Returns the token on every lane.
__device__ __forceinline__ int tree_pick_token(const float (&f)[4], int v, int V, double prefix, double target, double Z,
                                               uint32_t* flag) {
    const int lane = threadIdx.x & 63;
    const double l1 = (double)f[0], l2 = l1 + (double)f[1], l3 = l2 + (double)f[2], l4 = l3 + (double)f[3];
    const double base = prefix + (wave_inclusive_scan(l4) - l4);
    const double cdf[4] = {base + l1, base + l2, base + l3, base + l4};
    int hit = -1, lastlive = -1;
#pragma unroll
    for (int e = 3; e >= 0; --e) {
        if (f[e] > 0.f && cdf[e] > target) hit = e;
        if (lastlive < 0 && f[e] > 0.f) lastlive = e;
    }
    const unsigned long long cross = __ballot(hit >= 0);
    const unsigned long long live = __ballot(lastlive >= 0);
    int pick;
    if (cross) pick = __ffsll((long long)cross) - 1;
    else if (live) { pick = 63 - __clzll((long long)live); *flag |= TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE; }
    else { pick = 0; *flag |= TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE; }
    const int e = cross ? hit : (live ? lastlive : 0);
    int tok = v + e;
    uint32_t mine = 0;
    if (lane == pick) {
        const double tol = (double)kMargin * Z;
        const double fe = (double)(e == 0 ? f[0] : e == 1 ? f[1] : e == 2 ? f[2] : f[3]);
        const double hi_edge = e == 0 ? cdf[0] : e == 1 ? cdf[1] : e == 2 ? cdf[2] : cdf[3];
        if (fabs(hi_edge - target) < tol && tok + 1 < V) mine |= TABED_FLAG_SAMPLE_MARGIN;
        if (tok > 0 && fabs((hi_edge - fe) - target) < tol) mine |= TABED_FLAG_SAMPLE_MARGIN;
    }
    tok = tok < V ? tok : V - 1;
    *flag |= (uint32_t)__builtin_amdgcn_readlane((int)mine, pick);
    return __builtin_amdgcn_readlane(tok, pick);
}

template <bool VEC, int N>
__global__ __launch_bounds__(kBlock) void k_tree_level(TreeArgs a, int L) {
    const int c = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double* ts = a.tstate + (size_t)b * kTsSlots;
    if ((int)ts[kTsStatus] != kTreePending || (int)ts[kTsIndex] != L) return;      // uniform over the grid row
    const int V = a.V, n = (N > 0) ? N : a.n, gamma = a.gamma, S = a.S, NSEG = a.NSEG;
    const int k = (int)ts[kTsK];
    const float T = a.temperature[b];
    const double Z1 = ts[kTsZ1], Z2 = ts[kTsZ2];
    const float invZ1 = (float)(1.0 / Z1), invZ2 = (L >= 3) ? (float)(1.0 / Z2) : 0.f;

    __shared__ float s_hi[TABED_MAX_N], s_lo[TABED_MAX_N], s_w[TABED_MAX_N];
    __shared__ double s_redd[kWavesPerBlock];
    __shared__ int s_last, s_first[kWavesPerBlock], s_lastw[kWavesPerBlock], s_seg;
    __shared__ double s_prefix;
    if (tid < n) {
        const double l = a.dlse[((size_t)k * a.B + b) * n + tid];
        const float hi = (float)l;
        s_hi[tid] = hi;
        s_lo[tid] = (float)(1.0 - (l - (double)hi));
        s_w[tid] = a.weights[(size_t)b * n + tid];
    }
    __syncthreads();
    ResidRow r;
    r.bonus = false;
    r.invT = 1.f / T;
    r.trow = a.target + ((size_t)b * (gamma + 1) + k) * V;
    r.pmax = (float)ts[kTsRowMax];
    r.pinvZ = (float)(1.0 / ts[kTsRowZ]);
    r.qrows = a.dlogits + ((size_t)k * a.B + b) * n * V;
    // level L from the elementwise values: f_1 = max(0, p - q), f_2 = max(0, f_1 / Z_1 - q), f_3 = max(0, f_2 / Z_2 - q)
    auto level = [&](float f1, float q) {
        float f = fmaxf(0.f, f1 * invZ1 - q);
        if (L >= 3) f = fmaxf(0.f, f * invZ2 - q);
        return f;
    };
    constexpr int kSegPerChunk = kResidChunkV / kSegV, kSegPerWave = kSegPerChunk / kWavesPerBlock;
    {
        float f[kSegPerWave][4], p[kSegPerWave][4], q[kSegPerWave][4];
        int vs[kSegPerWave];
#pragma unroll
        for (int sg = 0; sg < kSegPerWave; ++sg) vs[sg] = (c * kSegPerChunk + wave + sg * kWavesPerBlock) * kSegV + lane * 4;
        resid_eval<VEC, N, kSegPerWave>(r, n, V, vs, s_hi, s_lo, s_w, f, p, q);
#pragma unroll
        for (int sg = 0; sg < kSegPerWave; ++sg) {
            const int seg = c * kSegPerChunk + wave + sg * kWavesPerBlock;
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) acc += level(f[sg][e], q[sg][e]);
            const double m = (double)wave_sum(acc);
            if (lane == 0 && seg < NSEG) publish_store(&a.tseg[((size_t)b * 2 + 0) * NSEG + seg], m);
        }
    }
    publish_barrier();
    if (tid == 0) s_last = arrive(&a.tickets[b], (uint32_t)a.C5) ? 1 : 0;
    __syncthreads();
    if (!s_last) return;

    // ---- last workgroup of the sequence: the level's mass, then sibling L's test or the corrected token
    const double* massL = a.tseg + ((size_t)b * 2 + 0) * NSEG;
    const double* massP = a.segP + ((size_t)b * 2 + 1) * NSEG;
    const int SPT = (NSEG + kBlock - 1) / kBlock;
    const int g0 = min(NSEG, tid * SPT), g1 = min(NSEG, g0 + SPT);
    double run = 0.0;
    for (int g = g0; g < g1; ++g) run += published_load(&massL[g]);
    double Z;
    double excl = block_exclusive_scan(run, s_redd, &Z);
    const size_t fidx = (size_t)b * (gamma + 1) + k;
    uint32_t flag = a.flags[fidx];
    const bool degenerate = !(Z > 0.0);
    const double* mass = massL;
    if (degenerate) {
        // empty residual (the lower level equals q): the token is drawn from p_k, whose segment masses the
        // chain's residual pass left behind
        flag |= TABED_FLAG_DEGENERATE;
        run = 0.0;
        for (int g = g0; g < g1; ++g) run += massP[g];
        excl = block_exclusive_scan(run, s_redd, &Z);
        mass = massP;
        r.bonus = true;
    } else if (L <= S) {
        if (tid == 0) {
            const size_t so = ((size_t)b * gamma + k) * S + (L - 1);
            const int y = a.sib_tokens[so];
            int decided = 0;
            if (y >= 0 && y < V) {
                const double lse = ts[kTsRowMax] + log(ts[kTsRowZ]);
                const double py = exp((double)(r.trow[y] * r.invT) - lse);
                const float u = a.u_acc_sib ? a.u_acc_sib[so]
                                            : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)k + (uint32_t)L * kSiblingStride, 1);
                if (tree_test(L, py, (double)a.sib_q[so], Z1, Z2, Z, u, &flag)) decided = 1;
            } else {
                flag |= TABED_FLAG_DEGENERATE;
            }
            a.flags[fidx] = (uint8_t)flag;
            if (decided) { ts[kTsStatus] = (double)kTreeLeaf; ts[kTsIndex] = (double)L; }
            else { ts[kTsIndex] = (double)(L + 1); ts[kTsZ2] = Z; }   // L = 2: widths above 3 would need a Z_3
        }
        return;                                            // the next pass continues (or the leaf's bonus pass)
    }
    const float u = a.u_res ? a.u_res[b] : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)gamma, 0);
    const double target = (double)u * Z;
    if (!tree_pick_segment(mass, g0, g1, excl, run, target, s_first, s_lastw, &s_seg, &s_prefix)) {
        if (tid == 0) {
            a.out_tokens[fidx] = 0;
            a.flags[fidx] = (uint8_t)(flag | TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE);
            ts[kTsStatus] = (double)kTreeDone;
        }
        return;
    }
    if (tid >= kWave) return;
    const int v1[1] = {s_seg * kSegV + lane * 4};
    float f1[1][4], p1[1][4], q1[1][4], fl[4];
    resid_eval<VEC, N, 1>(r, n, V, v1, s_hi, s_lo, s_w, f1, p1, q1);
#pragma unroll
    for (int e = 0; e < 4; ++e) fl[e] = degenerate ? p1[0][e] : level(f1[0][e], q1[0][e]);
    const int tok = tree_pick_token(fl, v1[0], V, s_prefix, target, Z, &flag);
    if (lane == 0) {
        a.out_tokens[fidx] = tok;
        a.flags[fidx] = (uint8_t)flag;
        ts[kTsStatus] = (double)kTreeDone;
    }
}

// Bonus token after an accepted leaf: a draw from softmax(leaf row / T) with the round's u_res (arg-max for a
// greedy row).  Every wave leaves, per 256-wide segment, the maximum of the scaled logits and the sum of
// exp(. - that maximum); the last workgroup combines them (fp64, segment order), finds the segment the uniform
// falls into and re-evaluates it.  Greedy: per-segment (value, index) arg-max records, merged lowest index first.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_tree_bonus(TreeArgs a) {
    const int c = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double* ts = a.tstate + (size_t)b * kTsSlots;
    if ((int)ts[kTsStatus] != kTreeLeaf) return;
    const int V = a.V, gamma = a.gamma, S = a.S, NSEG = a.NSEG;
    const int k = (int)ts[kTsK], sidx = (int)ts[kTsIndex];
    const float T = a.temperature[b];
    const bool greedy = !(T > 0.f);
    const float invT = greedy ? 1.f : 1.f / T;
    const size_t so = ((size_t)b * gamma + k) * S + (sidx - 1);
    const float* row = a.leaf_logits + so * V;
    double* rec0 = a.tseg + ((size_t)b * 2 + 0) * NSEG;    // sampling: segment sum;  greedy: arg-max value
    double* rec1 = a.tseg + ((size_t)b * 2 + 1) * NSEG;    // sampling: segment max;  greedy: arg-max index

    __shared__ double s_redd[kWavesPerBlock];
    __shared__ float s_redf[kWavesPerBlock];
    __shared__ ArgMax s_am[kWavesPerBlock];
    __shared__ int s_last, s_first[kWavesPerBlock], s_lastw[kWavesPerBlock], s_seg;
    __shared__ double s_prefix;

    constexpr int kSegPerChunk = kResidChunkV / kSegV, kSegPerWave = kSegPerChunk / kWavesPerBlock;
    float4 x[kSegPerWave];
#pragma unroll
    for (int sg = 0; sg < kSegPerWave; ++sg)
        x[sg] = load4<VEC>(row, (c * kSegPerChunk + wave + sg * kWavesPerBlock) * kSegV + lane * 4, V);
#pragma unroll
    for (int sg = 0; sg < kSegPerWave; ++sg) {
        const int seg = c * kSegPerChunk + wave + sg * kWavesPerBlock;
        const int v = seg * kSegV + lane * 4;
        if (greedy) {
            ArgMax am{-INFINITY, 0x7fffffff};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (v + e < V) am = argmax_merge(am, ArgMax{f4get(x[sg], e), v + e});
            am = wave_argmax(am);
            if (lane == 0 && seg < NSEG) { publish_store(&rec0[seg], (double)am.v); publish_store(&rec1[seg], (double)am.i); }
        } else {
            float mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < 4; ++e) mx = fmaxf(mx, f4get(x[sg], e) * invT);
            mx = wave_max(mx);
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float st = f4get(x[sg], e) * invT;
                if (st > -INFINITY) acc += __expf(st - mx);
            }
            const double sum = (double)wave_sum(acc);
            if (lane == 0 && seg < NSEG) { publish_store(&rec0[seg], sum); publish_store(&rec1[seg], (double)mx); }
        }
    }
    publish_barrier();
    if (tid == 0) s_last = arrive(&a.tickets[b], (uint32_t)a.C5) ? 1 : 0;
    __syncthreads();
    if (!s_last) return;

    const size_t fidx = (size_t)b * (gamma + 1) + k;
    const int SPT = (NSEG + kBlock - 1) / kBlock;
    const int g0 = min(NSEG, tid * SPT), g1 = min(NSEG, g0 + SPT);
    const int leaf_tok = a.sib_tokens[so];
    if (greedy) {
        ArgMax am{-INFINITY, 0x7fffffff};
        for (int g = g0; g < g1; ++g) am = argmax_merge(am, ArgMax{(float)published_load(&rec0[g]), (int)published_load(&rec1[g])});
        am = wave_argmax(am);
        if (lane == 0) s_am[wave] = am;
        __syncthreads();
        if (tid == 0) {
            ArgMax t = s_am[0];
            for (int w = 1; w < kWavesPerBlock; ++w) t = argmax_merge(t, s_am[w]);
            a.out_tokens[fidx] = leaf_tok;
            a.out_tokens[fidx + 1] = (t.i >= 0 && t.i < V) ? t.i : 0;
            a.flags[fidx + 1] = 0;
            a.leaf[b] = sidx;
            a.n_out[b] = k + 2;
            ts[kTsStatus] = (double)kTreeDone;
        }
        return;
    }
    float ml = -INFINITY;
    for (int g = g0; g < g1; ++g) ml = fmaxf(ml, (float)published_load(&rec1[g]));
    const float M = block_max(ml, s_redf);
    double run = 0.0;
    for (int g = g0; g < g1; ++g) {
        const double sg = published_load(&rec0[g]);
        if (sg > 0.0) run += sg * exp(published_load(&rec1[g]) - (double)M);
    }
    // rescaled masses go back to slot 0 so that the owner can walk its own run (only this workgroup is left)
    double Z;
    const double excl = block_exclusive_scan(run, s_redd, &Z);
    const float u = a.u_res ? a.u_res[b] : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)gamma, 0);
    const double target = (double)u * Z;
    uint32_t flag = 0;
    const int owner = block_find_owner(excl, run, target, s_first, s_lastw);
    if (owner < 0) {
        if (tid == 0) {
            a.out_tokens[fidx] = leaf_tok; a.out_tokens[fidx + 1] = 0;
            a.flags[fidx + 1] = (uint8_t)(TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE);
            a.leaf[b] = sidx; a.n_out[b] = k + 2; ts[kTsStatus] = (double)kTreeDone;
        }
        return;
    }
    if (tid == owner) {
        double P = excl, Plast = excl;
        int gstar = -1, glast = g0;
        for (int g = g0; g < g1; ++g) {
            const double sg = published_load(&rec0[g]);
            const double mg = (sg > 0.0) ? sg * exp(published_load(&rec1[g]) - (double)M) : 0.0;
            if (mg > 0.0) { glast = g; Plast = P; }
            if (P + mg > target) { gstar = g; break; }
            P += mg;
        }
        if (gstar < 0) { gstar = glast; P = Plast; }
        s_seg = gstar;
        s_prefix = P;
    }
    __syncthreads();
    if (tid >= kWave) return;
    const int v = s_seg * kSegV + lane * 4;
    const float4 xx = load4<VEC>(row, v, V);
    float f[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float st = f4get(xx, e) * invT;
        f[e] = (st > -INFINITY) ? __expf(st - M) : 0.f;
    }
    const int tok = tree_pick_token(f, v, V, s_prefix, target, Z, &flag);
    if (lane == 0) {
        a.out_tokens[fidx] = leaf_tok;
        a.out_tokens[fidx + 1] = tok;
        a.flags[fidx + 1] = (uint8_t)flag;
        a.leaf[b] = sidx;
        a.n_out[b] = k + 2;
        ts[kTsStatus] = (double)kTreeDone;
    }
}

hipError_t launch_verify_tree(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round, int width,
                              const float* target_logits, const float* leaf_logits, const float* draft_logits,
                              const double* draft_lse, const int32_t* sib_tokens, const float* sib_q,
                              const float* weights, const float* temperature, const float* u_res,
                              const float* u_acc_sib, int32_t* out_tokens, uint8_t* flags, int32_t* leaf,
                              int32_t* n_out, hipStream_t s) {
    ProfScope prof(TABED_K_TREE, s);
    TreeArgs a;
    a.V = c.V; a.n = c.n; a.B = c.B; a.gamma = c.gamma; a.S = width - 1; a.NSEG = L.NSEG; a.C5 = L.C5;
    a.seed = c.seed; a.round = round;
    a.target = target_logits; a.leaf_logits = leaf_logits; a.dlogits = draft_logits; a.dlse = draft_lse;
    a.sib_tokens = sib_tokens; a.sib_q = sib_q; a.weights = weights; a.temperature = temperature;
    a.u_res = u_res; a.u_acc_sib = u_acc_sib;
    a.tstate = reinterpret_cast<double*>(ws + L.off_tstate);
    a.segP = reinterpret_cast<const double*>(ws + L.off_seg);
    a.tseg = reinterpret_cast<double*>(ws + L.off_tseg);
    a.out_tokens = out_tokens; a.flags = flags; a.leaf = leaf; a.n_out = n_out;
    a.tickets = reinterpret_cast<uint32_t*>(ws + L.off_tickets) + 3 * c.B;
    // sibling 1 against the first residual (its mass is known from tabed_verify's pass); width 1: leaf = 0, n_out = k + 1
    launch(&prof, k_tree_begin, dim3(c.B), dim3(64), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || width == 1) return e;
    const bool vec = (c.V % 4 == 0);
    const int ncomp = (vec && (c.n == 2 || c.n == 4 || c.n == 8)) ? c.n : 0;
    const dim3 grid(L.C5, c.B);
    for (int lvl = 2; lvl <= width; ++lvl) {
        if (!vec) launch(nullptr, k_tree_level<false, 0>, grid, dim3(kBlock), 0, s, a, lvl);
        else if (ncomp == 2) launch(nullptr, k_tree_level<true, 2>, grid, dim3(kBlock), 0, s, a, lvl);
        else if (ncomp == 4) launch(nullptr, k_tree_level<true, 4>, grid, dim3(kBlock), 0, s, a, lvl);
        else if (ncomp == 8) launch(nullptr, k_tree_level<true, 8>, grid, dim3(kBlock), 0, s, a, lvl);
        else launch(nullptr, k_tree_level<true, 0>, grid, dim3(kBlock), 0, s, a, lvl);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    a.tickets = reinterpret_cast<uint32_t*>(ws + L.off_tickets) + 4 * c.B;
    if (vec) launch(nullptr, k_tree_bonus<true>, grid, dim3(kBlock), 0, s, a);
    else launch(nullptr, k_tree_bonus<false>, grid, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace tabed
