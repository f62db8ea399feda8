// Vocabulary-wide passes of a TABED round on gfx950: ensemble + draft token (Alg. 1 lines 6-7),
// target statistics + per-draft KL + accept chain (Sec. 3 items 2-3, Sec. 4.1), corrected / bonus token
// (Sec. 3 item 3), window + weights (Alg. 1 lines 2-3, App. B.2).  All of them are HBM- or latency-bound:
// wave64 shuffles and a few LDS words do the reductions, fp64 carries every cross-lane sum.
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
    const int count = 3 * c.B;
    hipLaunchKernelGGL(k_fill_u32, dim3((count + 255) / 256), dim3(256), 0, s,
                       reinterpret_cast<uint32_t*>(ws + L.off_tickets), count);
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
    hipLaunchKernelGGL(k_philox, dim3((count + 255) / 256), dim3(256), 0, s, c.seed, round, c.B, c.gamma + 1, out);
    return hipGetLastError();
}

// One thread per sequence: push the verified positions into the window, sum it, softmax of 1/e.
// Everything after the fp32 loads is fp64: B*n scalars, latency-bound.
__global__ void k_weights(int n, int B, int gamma, int h, int policy, double tau_w, double eps,
                          const float* __restrict__ dev, const int32_t* __restrict__ n_valid,
                          float* ring, int32_t* ring_head, int32_t* ring_count, float* weights) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int head = ring_head[b], count = ring_count[b];
    head = ((head % h) + h) % h;
    count = count < 0 ? 0 : (count > h ? h : count);
    float* rb = ring + (size_t)b * h * n;
    if (dev != nullptr && n_valid != nullptr) {
        int nv = n_valid[b];
        nv = nv < 0 ? 0 : (nv > gamma ? gamma : nv);
        for (int i = 0; i < nv; ++i) {
            for (int j = 0; j < n; ++j) rb[(size_t)head * n + j] = dev[((size_t)b * gamma + i) * n + j];
            head = (head + 1) % h;
            if (count < h) ++count;
        }
        ring_head[b] = head;
        ring_count[b] = count;
    }
    float* w = weights + (size_t)b * n;
    if (policy == 1 || count == 0) {
        const float eq = (float)(1.0 / (double)n);
        for (int j = 0; j < n; ++j) w[j] = eq;
        return;
    }
    double x[TABED_MAX_N];
    double xmax = -INFINITY;
    for (int j = 0; j < n; ++j) {
        double e = 0.0;
        for (int t = 0; t < count; ++t) {            // oldest .. newest
            const int slot = ((head - count + t) % h + h) % h;
            e += (double)rb[(size_t)slot * n + j];
        }
        x[j] = (1.0 / fmax(e, eps)) / tau_w;
        xmax = fmax(xmax, x[j]);
    }
    double Z = 0.0;
    for (int j = 0; j < n; ++j) { x[j] = exp(x[j] - xmax); Z += x[j]; }
    for (int j = 0; j < n; ++j) w[j] = (float)(x[j] / Z);
}

hipError_t launch_weights(const tabed_cfg& c, const float* dev, const int32_t* n_valid, float* ring,
                          int32_t* ring_head, int32_t* ring_count, float* weights, hipStream_t s) {
    ProfScope prof(TABED_K_WEIGHTS, s);
    hipLaunchKernelGGL(k_weights, dim3((c.B + 63) / 64), dim3(64), 0, s, c.n, c.B, c.gamma, c.h, c.policy,
                       (double)c.tau_w, (double)c.eps, dev, n_valid, ring, ring_head, ring_count, weights);
    return hipGetLastError();
}

// =====================================================================================================
// Ensemble + draft token.
// The LM-head epilogue left, per draft row and per 32-wide vocabulary tile, the tile maximum of the scaled
// logits and the tile sum of exp(scaled logit - tile maximum).  From those alone this kernel gets every
// draft's log-sum-exp and the mass of the mixture q = sum_j w_j q^(j) inside every tile; a sampling row
// therefore reads logits only inside the one tile its uniform falls into.  A greedy row needs the arg-max
// of q over the whole vocabulary: its row is split over gridDim.x workgroups and the last one to arrive
// merges the candidates in chunk order.
// =====================================================================================================
struct SampleArgs {
    int V, n, B, gamma, pos, NT, C2;
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

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_sample(SampleArgs a) {
    const int b = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
    const int n = a.n, NT = a.NT, V = a.V;
    const float T = a.temperature[b];
    const bool greedy = !(T > 0.f);
    if (!greedy && c != 0) return;
    const float invT = greedy ? 1.f : 1.f / T;

    __shared__ float s_m[TABED_MAX_N];    // row maximum of scaled logits
    __shared__ double s_c[TABED_MAX_N];   // w_j / sum_v exp(scaled - max)
    __shared__ float s_cf[TABED_MAX_N];
    __shared__ float s_redf[kWavesPerBlock];
    __shared__ double s_redd[kWavesPerBlock];
    __shared__ int s_owner, s_fallback, s_tile, s_last;
    __shared__ double s_prefix;
    __shared__ Top2 s_top[kWavesPerBlock];

    // ---- per-draft log-sum-exp from the tile partials
    for (int j = 0; j < n; ++j) {
        const float* pmr = a.pm + (size_t)(b * n + j) * NT;
        const float* psr = a.ps + (size_t)(b * n + j) * NT;
        float m = -INFINITY;
        for (int t = tid; t < NT; t += kBlock) m = fmaxf(m, pmr[t]);
        m = block_max(m, s_redf);
        double s = 0.0;
        for (int t = tid; t < NT; t += kBlock) s += (double)(psr[t] * __expf(pmr[t] - m));
        s = block_sum(s, s_redd);
        if (tid == 0) {
            s_m[j] = m;
            s_c[j] = (double)a.weights[(size_t)b * n + j] / s;
            s_cf[j] = (float)s_c[j];
            if (c == 0) a.draft_lse[((size_t)a.pos * a.B + b) * n + j] = (double)m + log(s);
        }
    }
    if (tid == 0) { s_owner = kBlock; s_fallback = -1; }
    __syncthreads();

    const float* rows = a.logits + (size_t)b * n * V;
    const size_t out_idx = (size_t)b * a.gamma + a.pos;

    if (!greedy) {
        // ---- tile masses of the mixture, thread-contiguous runs of tiles, fixed-order prefix
        const int S = (NT + kBlock - 1) / kBlock;
        const int t0 = min(NT, tid * S), t1 = min(NT, t0 + S);
        auto tile_mass = [&](int t) -> double {
            double acc = 0.0;
            for (int j = 0; j < n; ++j) {
                const size_t o = (size_t)(b * n + j) * NT + t;
                acc += s_c[j] * (double)(a.ps[o] * __expf(a.pm[o] - s_m[j]));
            }
            return acc;
        };
        double run = 0.0;
        for (int t = t0; t < t1; ++t) run += tile_mass(t);
        double Z;
        const double excl = block_exclusive_scan(run, s_redd, &Z);
        const float u = a.u_draft ? a.u_draft[out_idx] : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)a.pos, 0);
        const double target = (double)u * Z;
        if (run > 0.0) {
            if (excl + run > target) atomicMin(&s_owner, tid);
            atomicMax(&s_fallback, tid);
        }
        __syncthreads();
        const int owner = s_owner < kBlock ? s_owner : s_fallback;   // -1 only if every mass is zero
        if (owner < 0) {
            if (tid == 0) {
                a.draft_tokens[out_idx] = 0;
                a.draft_q[out_idx] = 0.f;
                a.flags[out_idx] = (uint8_t)(TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE);
            }
            return;
        }
        if (tid == owner) {
            double P = excl;
            int tstar = -1, tlast = t0;
            double Plast = excl;
            for (int t = t0; t < t1; ++t) {
                const double mt = tile_mass(t);
                if (mt > 0.0) { tlast = t; Plast = P; }
                if (P + mt > target) { tstar = t; break; }
                P += mt;
            }
            if (tstar < 0) { tstar = tlast; P = Plast; }
            s_tile = tstar;
            s_prefix = P;
        }
        __syncthreads();
        if (tid >= kWave) return;
        // ---- wave 0 resolves the token inside the tile
        const int lane = tid, v = s_tile * kTileV + lane;
        double f = 0.0;
        if (lane < kTileV && v < V)
            for (int j = 0; j < n; ++j) f += s_c[j] * (double)__expf(rows[(size_t)j * V + v] * invT - s_m[j]);
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
    Top2 best = top2_empty();
    const int cb = c * kChunkV;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int v = cb + (u * kBlock + tid) * 4;
        if (v >= V) continue;
        float q[4] = {0.f, 0.f, 0.f, 0.f};
        for (int j = 0; j < n; ++j) {
            const float4 x = load4<VEC>(rows + (size_t)j * V, v, V);
            const float cj = s_cf[j], mj = s_m[j];
            q[0] += cj * __expf(x.x * invT - mj);
            q[1] += cj * __expf(x.y * invT - mj);
            q[2] += cj * __expf(x.z * invT - mj);
            q[3] += cj * __expf(x.w * invT - mj);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (v + e < V) best = top2_push(best, q[e], v + e);
    }
    best = wave_top2(best);
    if ((tid & 63) == 0) s_top[tid >> 6] = best;
    __syncthreads();
    if (tid == 0) {
        Top2 t = s_top[0];
        for (int w = 1; w < kWavesPerBlock; ++w) t = top2_merge(t, s_top[w]);
        a.cand[(size_t)b * a.C2 + c] = Top2Rec{t.v1, t.i1, t.v2, 0};
        __threadfence();
        const uint32_t old = atomicAdd(&a.tickets[b], 1u);
        s_last = (old == (uint32_t)(a.C2 - 1));
    }
    __syncthreads();
    if (!s_last || tid != 0) return;
    __threadfence();
    Top2 t = top2_empty();
    for (int cc = 0; cc < a.C2; ++cc) {
        const Top2Rec r = a.cand[(size_t)b * a.C2 + cc];
        t = top2_merge(t, Top2{r.v1, r.i1, r.v2});
    }
    a.tickets[b] = 0u;
    const int y = (t.i1 >= 0 && t.i1 < V) ? t.i1 : 0;
    double f = 0.0;
    for (int j = 0; j < n; ++j) f += s_c[j] * (double)__expf(rows[(size_t)j * V + y] * invT - s_m[j]);
    uint32_t flag = 0;
    if (V > 1 && (t.v1 - t.v2) < kMargin * fabsf(t.v1)) flag |= TABED_FLAG_SAMPLE_MARGIN;
    a.draft_tokens[out_idx] = y;
    a.draft_q[out_idx] = (float)f;
    a.flags[out_idx] = (uint8_t)flag;
}

hipError_t launch_sample(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round, int pos,
                         const float* logits, const float* weights, const float* temperature,
                         const float* u_draft, double* draft_lse, int32_t* draft_tokens, float* draft_q,
                         uint8_t* flags, hipStream_t s) {
    ProfScope prof(TABED_K_SAMPLE, s);
    SampleArgs a;
    a.V = c.V; a.n = c.n; a.B = c.B; a.gamma = c.gamma; a.pos = pos; a.NT = L.NT; a.C2 = L.C2;
    a.seed = c.seed; a.round = round;
    a.logits = logits;
    a.pm = reinterpret_cast<const float*>(ws + L.off_pm);
    a.ps = reinterpret_cast<const float*>(ws + L.off_ps);
    a.weights = weights; a.temperature = temperature; a.u_draft = u_draft;
    a.draft_lse = draft_lse; a.draft_tokens = draft_tokens; a.draft_q = draft_q; a.flags = flags;
    a.cand = reinterpret_cast<Top2Rec*>(ws + L.off_cand);
    a.tickets = reinterpret_cast<uint32_t*>(ws + L.off_tickets) + 0 * c.B;
    const dim3 grid(L.C2, c.B);
    if (c.V % 4 == 0) hipLaunchKernelGGL(k_sample<true>, grid, dim3(kBlock), 0, s, a);
    else              hipLaunchKernelGGL(k_sample<false>, grid, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

// =====================================================================================================
// Target statistics, per-draft KL, accept chain.
// Grid (chunk, position i <= gamma, sequence b).  Each workgroup reads its chunk of the target row once,
// and for i < gamma the same chunk of the n draft rows once, and leaves a record
//   { m_c = max scaled target logit, Z_c = sum exp(st - m_c), arg-max of the raw row,
//     A_jc = sum exp(st - m_c) * (st - s_j)  for every draft j }.
// Since KL(p || q_j) = sum_v p (st - s_j) - lse_p + lse_j, these records combine exactly (in fp64, in chunk
// order) once all chunks of a sequence have arrived; the last workgroup of a sequence does that and then
// walks the accept chain of Sec. 3 item 3.
// =====================================================================================================
struct StatsArgs {
    int V, n, B, gamma, C3, RS;
    uint64_t seed, round;
    const float* target;
    const float* dlogits;
    const double* dlse;
    const int32_t* dtok;
    const float* dq;
    const float* temperature;
    const float* u_acc;
    double* stats;
    double* lsep;   // [B][gamma+1][2]: row maximum, 1 / sum exp(st - max)
    int32_t* amax;
    uint32_t* tickets;
    int32_t* accept_len;
    int32_t* out_tokens;
    float* dev;
    int32_t* n_valid;
    uint8_t* flags;
};

template <bool VEC, int U>
__global__ __launch_bounds__(kBlock) void k_stats(StatsArgs a) {
    const int c = blockIdx.x, i = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int V = a.V, n = a.n, gamma = a.gamma;
    const float T = a.temperature[b];
    const bool greedy = !(T > 0.f);
    const float invT = greedy ? 1.f : 1.f / T;

    __shared__ float s_redf[kWavesPerBlock];
    __shared__ double s_redd[kWavesPerBlock];
    __shared__ ArgMax s_am[kWavesPerBlock];
    __shared__ double s_A[kWavesPerBlock][TABED_MAX_N];
    __shared__ int s_last;

    const float* trow = a.target + ((size_t)b * (gamma + 1) + i) * V;
    const int cb = c * (kBlock * 4 * U);
    float st[U * 4], ex[U * 4];
    ArgMax am{-INFINITY, 0x7fffffff};
    float tmax = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int v = cb + (u * kBlock + tid) * 4;
        const float4 x = load4<VEC>(trow, v, V);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float xe = f4get(x, e);
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
    const double Zc = block_sum((double)zf, s_redd);
    am = wave_argmax(am);
    if ((tid & 63) == 0) s_am[tid >> 6] = am;

    if (i < gamma) {
        for (int j = 0; j < n; ++j) {
            const float* qrow = a.dlogits + (((size_t)i * a.B + b) * n + j) * V;
            float aj = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int v = cb + (u * kBlock + tid) * 4;
                const float4 y = load4<VEC>(qrow, v, V);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float p = ex[u * 4 + e];
                    if (p > 0.f) aj += p * (st[u * 4 + e] - f4get(y, e) * invT);
                }
            }
            const double Aj = wave_sum((double)aj);
            if ((tid & 63) == 0) s_A[tid >> 6][j] = Aj;
        }
    }
    __syncthreads();
    double* rec = a.stats + (((size_t)b * (gamma + 1) + i) * a.C3 + c) * a.RS;
    if (tid == 0) {
        ArgMax t = s_am[0];
        for (int w = 1; w < kWavesPerBlock; ++w) t = argmax_merge(t, s_am[w]);
        rec[0] = (double)mc;
        rec[1] = Zc;
        rec[2] = (double)t.v;
        rec[3] = (double)t.i;
    }
    if (i < gamma && tid < n) rec[kStatHdr + tid] = (s_A[0][tid] + s_A[1][tid]) + (s_A[2][tid] + s_A[3][tid]);
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t old = atomicAdd(&a.tickets[b], 1u);
        s_last = (old == (uint32_t)((gamma + 1) * a.C3 - 1));
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();

    // ---- last workgroup of sequence b: combine chunks, distances, accept chain
    __shared__ double s_rowm[TABED_MAX_GAMMA + 1], s_rowZ[TABED_MAX_GAMMA + 1], s_rowlse[TABED_MAX_GAMMA + 1];
    __shared__ int s_rowam[TABED_MAX_GAMMA + 1];
    const double* sb = a.stats + (size_t)b * (gamma + 1) * a.C3 * a.RS;
    if (tid <= gamma) {
        const double* r0 = sb + (size_t)tid * a.C3 * a.RS;
        double m = -INFINITY;
        for (int cc = 0; cc < a.C3; ++cc) m = fmax(m, r0[(size_t)cc * a.RS]);
        double Z = 0.0, bv = -INFINITY;
        int bi = 0;
        for (int cc = 0; cc < a.C3; ++cc) {
            const double* r = r0 + (size_t)cc * a.RS;
            if (r[0] > -INFINITY) Z += r[1] * exp(r[0] - m);
            if (r[2] > bv) { bv = r[2]; bi = (int)r[3]; }   // chunk order: ties keep the lowest index
        }
        s_rowm[tid] = m; s_rowZ[tid] = Z; s_rowlse[tid] = m + log(Z); s_rowam[tid] = bi;
        a.lsep[((size_t)b * (gamma + 1) + tid) * 2 + 0] = m;
        a.lsep[((size_t)b * (gamma + 1) + tid) * 2 + 1] = 1.0 / Z;
        a.amax[(size_t)b * (gamma + 1) + tid] = bi;
    }
    __syncthreads();
    for (int q = tid; q < gamma * n; q += kBlock) {
        const int ii = q / n, j = q % n;
        const double* r0 = sb + (size_t)ii * a.C3 * a.RS;
        double A = 0.0;
        for (int cc = 0; cc < a.C3; ++cc) {
            const double* r = r0 + (size_t)cc * a.RS;
            if (r[0] > -INFINITY) A += r[kStatHdr + j] * exp(r[0] - s_rowm[ii]);
        }
        const double kl = A / s_rowZ[ii] - s_rowlse[ii] + a.dlse[((size_t)ii * a.B + b) * n + j];
        a.dev[((size_t)b * gamma + ii) * n + j] = (float)kl;
    }
    if (tid != 0) return;
    a.tickets[b] = 0u;
    int k = 0;
    bool open = true;
    for (int ii = 0; ii < gamma; ++ii) {
        uint32_t flag = 0;
        if (open) {
            const int y = a.dtok[(size_t)b * gamma + ii];
            bool ok;
            if (y < 0 || y >= V) { ok = false; flag |= TABED_FLAG_DEGENERATE; }
            else if (greedy) ok = (y == s_rowam[ii]);
            else {
                const float u = a.u_acc ? a.u_acc[(size_t)b * gamma + ii]
                                        : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)ii, 1);
                const float sty = a.target[((size_t)b * (gamma + 1) + ii) * V + y] * invT;
                const float py = (float)exp((double)sty - s_rowlse[ii]);
                const float lhs = u * a.dq[(size_t)b * gamma + ii];
                ok = lhs < py;
                if (fabs((double)lhs - (double)py) < (double)kMargin * fmax((double)lhs, (double)py))
                    flag |= TABED_FLAG_ACCEPT_MARGIN;
            }
            if (ok) ++k; else open = false;
        }
        a.flags[(size_t)b * (gamma + 1) + ii] = (uint8_t)flag;
    }
    a.flags[(size_t)b * (gamma + 1) + gamma] = 0;
    for (int ii = 0; ii <= gamma; ++ii)
        a.out_tokens[(size_t)b * (gamma + 1) + ii] = ii < k ? a.dtok[(size_t)b * gamma + ii] : -1;
    a.accept_len[b] = k;
    a.n_valid[b] = k + 1 < gamma ? k + 1 : gamma;
}

static int pick_stats_unroll(const tabed_cfg& c) {
    // Largest chunk that still gives the chip a few workgroups per compute unit.
    const long rows = (long)c.B * (c.gamma + 1);
    for (int U : {4, 2}) {
        const long chunks = (c.V + kBlock * 4 * U - 1) / (kBlock * 4 * U);
        if (rows * chunks >= 512) return U;
    }
    return 1;
}

hipError_t launch_stats(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round,
                        const float* target_logits, const float* draft_logits, const double* draft_lse,
                        const int32_t* draft_tokens, const float* draft_q, const float* temperature,
                        const float* u_acc, int32_t* accept_len, int32_t* out_tokens, float* dev,
                        int32_t* n_valid, uint8_t* flags, hipStream_t s) {
    ProfScope prof(TABED_K_STATS, s);
    const int U = pick_stats_unroll(c);
    StatsArgs a;
    a.V = c.V; a.n = c.n; a.B = c.B; a.gamma = c.gamma; a.RS = L.RS;
    a.C3 = (c.V + kBlock * 4 * U - 1) / (kBlock * 4 * U);
    a.seed = c.seed; a.round = round;
    a.target = target_logits; a.dlogits = draft_logits; a.dlse = draft_lse; a.dtok = draft_tokens;
    a.dq = draft_q; a.temperature = temperature; a.u_acc = u_acc;
    a.stats = reinterpret_cast<double*>(ws + L.off_stats);
    a.lsep = reinterpret_cast<double*>(ws + L.off_lsep);
    a.amax = reinterpret_cast<int32_t*>(ws + L.off_amax);
    a.tickets = reinterpret_cast<uint32_t*>(ws + L.off_tickets) + 1 * c.B;
    a.accept_len = accept_len; a.out_tokens = out_tokens; a.dev = dev; a.n_valid = n_valid; a.flags = flags;
    const dim3 grid(a.C3, c.gamma + 1, c.B);
    const bool vec = (c.V % 4 == 0);
#define TABED_LAUNCH_STATS(VEC_, U_) hipLaunchKernelGGL((k_stats<VEC_, U_>), grid, dim3(kBlock), 0, s, a)
    if (vec) { if (U == 4) TABED_LAUNCH_STATS(true, 4); else if (U == 2) TABED_LAUNCH_STATS(true, 2); else TABED_LAUNCH_STATS(true, 1); }
    else     { if (U == 4) TABED_LAUNCH_STATS(false, 4); else if (U == 2) TABED_LAUNCH_STATS(false, 2); else TABED_LAUNCH_STATS(false, 1); }
#undef TABED_LAUNCH_STATS
    return hipGetLastError();
}

// =====================================================================================================
// Corrected / bonus token.
// For a sampling row with k accepted tokens the emitted token comes from f = max(0, p_k - q_k) (k < gamma)
// or f = p_gamma (k = gamma).  Every wave writes the mass of f over its 256-wide segments; the last
// workgroup of the sequence prefixes the segment masses in order, finds the segment the uniform falls
// into, and one wave re-evaluates that segment element by element.  A greedy row just emits the arg-max
// of target row k found by the statistics kernel.
// =====================================================================================================
struct ResidArgs {
    int V, n, B, gamma, NSEG, C5;
    uint64_t seed, round;
    const float* target;
    const float* dlogits;
    const double* dlse;
    const float* weights;
    const float* temperature;
    const float* u_res;
    const int32_t* accept_len;
    const double* lsep;
    const int32_t* amax;
    double* seg;          // [B][2][NSEG]
    uint32_t* tickets;
    int32_t* out_tokens;
    uint8_t* flags;
};

// exp(x - (hi + lo)) with the rounding error of x - hi carried into a first-order correction, so that a
// log-sum-exp of magnitude ~10 does not cost the last three bits of the argument.
__device__ __forceinline__ float exp_shifted(float x, float hi, float lo) {
    const float s = x - hi;
    const float err = x - (s + hi);
    return expf(s) * (1.0f + (err - lo));
}

struct ResidRow {
    const float* trow;
    const float* qrows;   // n rows, stride V
    float invT, pmax, pinvZ;
    bool bonus;
};

// f and p for the four elements starting at v (v % 4 == 0).
template <bool VEC>
__device__ __forceinline__ void resid_elems(const ResidRow& r, int n, int V, int v, const float* s_hi,
                                            const float* s_lo, const float* s_w, float f[4], float p[4]) {
    const float4 x = load4<VEC>(r.trow, v, V);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float xe = f4get(x, e);
        p[e] = (v + e < V && xe > -INFINITY) ? expf(xe * r.invT - r.pmax) * r.pinvZ : 0.f;
    }
    if (r.bonus) {
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = p[e];
        return;
    }
    float q[4] = {0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < n; ++j) {
        const float4 y = load4<VEC>(r.qrows + (size_t)j * V, v, V);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float ye = f4get(y, e);
            if (v + e < V && ye > -INFINITY) q[e] += s_w[j] * exp_shifted(ye * r.invT, s_hi[j], s_lo[j]);
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) f[e] = fmaxf(0.f, p[e] - q[e]);
}

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_resid(ResidArgs a) {
    const int c = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = a.V, n = a.n, gamma = a.gamma, NSEG = a.NSEG;
    const float T = a.temperature[b];
    const bool greedy = !(T > 0.f);
    int k = a.accept_len[b];
    k = k < 0 ? 0 : (k > gamma ? gamma : k);
    const size_t out_idx = (size_t)b * (gamma + 1) + k;
    if (greedy) {
        if (c == 0 && tid == 0) a.out_tokens[out_idx] = a.amax[out_idx];
        return;
    }
    __shared__ float s_hi[TABED_MAX_N], s_lo[TABED_MAX_N], s_w[TABED_MAX_N];
    __shared__ double s_redd[kWavesPerBlock];
    __shared__ int s_last, s_owner, s_fallback, s_seg;
    __shared__ double s_prefix;

    ResidRow r;
    r.bonus = (k == gamma);
    r.invT = 1.f / T;
    r.trow = a.target + out_idx * V;
    r.pmax = (float)a.lsep[out_idx * 2 + 0];
    r.pinvZ = (float)a.lsep[out_idx * 2 + 1];
    r.qrows = r.bonus ? nullptr : a.dlogits + ((size_t)k * a.B + b) * n * V;
    if (tid < n && !r.bonus) {
        const double l = a.dlse[((size_t)k * a.B + b) * n + tid];
        s_hi[tid] = (float)l;
        s_lo[tid] = (float)(l - (double)s_hi[tid]);
        s_w[tid] = a.weights[(size_t)b * n + tid];
    }
    if (tid == 0) { s_owner = kBlock; s_fallback = -1; }
    __syncthreads();

    double* segR = a.seg + ((size_t)b * 2 + 0) * NSEG;
    double* segP = a.seg + ((size_t)b * 2 + 1) * NSEG;
    constexpr int kSegPerChunk = kChunkV / kSegV;
    for (int sidx = wave; sidx < kSegPerChunk; sidx += kWavesPerBlock) {
        const int seg = c * kSegPerChunk + sidx;
        if (seg >= NSEG) break;
        const int v = seg * kSegV + lane * 4;
        float f[4] = {0.f, 0.f, 0.f, 0.f}, p[4] = {0.f, 0.f, 0.f, 0.f};
        if (v < V) resid_elems<VEC>(r, n, V, v, s_hi, s_lo, s_w, f, p);
        const double mf = wave_sum((double)((f[0] + f[1]) + (f[2] + f[3])));
        const double mp = wave_sum((double)((p[0] + p[1]) + (p[2] + p[3])));
        if (lane == 0) { segR[seg] = mf; segP[seg] = mp; }
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t old = atomicAdd(&a.tickets[b], 1u);
        s_last = (old == (uint32_t)(a.C5 - 1));
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    if (tid == 0) a.tickets[b] = 0u;

    // ---- last workgroup of sequence b: locate the segment, then the token
    const int S = (NSEG + kBlock - 1) / kBlock;
    const int g0 = min(NSEG, tid * S), g1 = min(NSEG, g0 + S);
    uint32_t flag = 0;
    const double* mass = segR;
    if (!r.bonus) {
        double run = 0.0;
        for (int g = g0; g < g1; ++g) run += segR[g];
        const double Zr = block_sum(run, s_redd);
        if (!(Zr > 0.0)) { mass = segP; r.bonus = true; flag |= TABED_FLAG_DEGENERATE; }   // empty residual: draw from p_k
    }
    double run = 0.0;
    for (int g = g0; g < g1; ++g) run += mass[g];
    double Z;
    const double excl = block_exclusive_scan(run, s_redd, &Z);
    const float u = a.u_res ? a.u_res[b] : tabed_uniform(a.seed, a.round, (uint32_t)b, (uint32_t)gamma, 0);
    const double target = (double)u * Z;
    if (run > 0.0) {
        if (excl + run > target) atomicMin(&s_owner, tid);
        atomicMax(&s_fallback, tid);
    }
    __syncthreads();
    const int owner = s_owner < kBlock ? s_owner : s_fallback;
    if (owner < 0) {
        if (tid == 0) {
            a.out_tokens[out_idx] = 0;
            a.flags[out_idx] |= (uint8_t)(TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE);
        }
        return;
    }
    if (tid == owner) {
        double P = excl, Plast = excl;
        int gstar = -1, glast = g0;
        for (int g = g0; g < g1; ++g) {
            const double mg = mass[g];
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
    float f[4] = {0.f, 0.f, 0.f, 0.f}, p[4] = {0.f, 0.f, 0.f, 0.f};
    if (v < V) resid_elems<VEC>(r, n, V, v, s_hi, s_lo, s_w, f, p);
    const double l1 = (double)f[0], l2 = l1 + (double)f[1], l3 = l2 + (double)f[2], l4 = l3 + (double)f[3];
    const double base = s_prefix + (wave_inclusive_scan(l4) - l4);
    const double cdf[4] = {base + l1, base + l2, base + l3, base + l4};
    int hit = -1, lastlive = -1;
#pragma unroll
    for (int e = 3; e >= 0; --e) {
        if (f[e] > 0.f && cdf[e] > target) hit = e;
        if (lastlive < 0 && f[e] > 0.f) lastlive = e;
    }
    const unsigned long long cross = __ballot(hit >= 0);
    const unsigned long long live = __ballot(lastlive >= 0);
    int pick, e;
    if (cross) { pick = __ffsll((long long)cross) - 1; e = hit; }
    else if (live) { pick = 63 - __clzll((long long)live); e = lastlive; flag |= TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE; }
    else { pick = 0; e = 0; flag |= TABED_FLAG_SAMPLE_MARGIN | TABED_FLAG_DEGENERATE; }
    if (lane == pick) {
        const int tok = v + e;
        const double tol = (double)kMargin * Z;
        const double hi_edge = cdf[e], lo_edge = cdf[e] - (double)f[e];
        if (fabs(hi_edge - target) < tol && tok + 1 < V) flag |= TABED_FLAG_SAMPLE_MARGIN;
        if (tok > 0 && fabs(lo_edge - target) < tol) flag |= TABED_FLAG_SAMPLE_MARGIN;
        a.out_tokens[out_idx] = tok < V ? tok : V - 1;
        a.flags[out_idx] |= (uint8_t)flag;
    }
}

hipError_t launch_resid(const tabed_cfg& c, const WsLayout& L, char* ws, uint64_t round,
                        const float* target_logits, const float* draft_logits, const double* draft_lse,
                        const float* weights, const float* temperature, const float* u_res,
                        const int32_t* accept_len, int32_t* out_tokens, uint8_t* flags, hipStream_t s) {
    ProfScope prof(TABED_K_RESID, s);
    ResidArgs a;
    a.V = c.V; a.n = c.n; a.B = c.B; a.gamma = c.gamma; a.NSEG = L.NSEG; a.C5 = L.C5;
    a.seed = c.seed; a.round = round;
    a.target = target_logits; a.dlogits = draft_logits; a.dlse = draft_lse; a.weights = weights;
    a.temperature = temperature; a.u_res = u_res; a.accept_len = accept_len;
    a.lsep = reinterpret_cast<const double*>(ws + L.off_lsep);
    a.amax = reinterpret_cast<const int32_t*>(ws + L.off_amax);
    a.seg = reinterpret_cast<double*>(ws + L.off_seg);
    a.tickets = reinterpret_cast<uint32_t*>(ws + L.off_tickets) + 2 * c.B;
    a.out_tokens = out_tokens; a.flags = flags;
    const dim3 grid(L.C5, c.B);
    if (c.V % 4 == 0) hipLaunchKernelGGL(k_resid<true>, grid, dim3(kBlock), 0, s, a);
    else              hipLaunchKernelGGL(k_resid<false>, grid, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace tabed
