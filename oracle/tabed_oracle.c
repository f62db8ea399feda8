/*
 * TABED per-round hot path -- plain CPU oracle.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT.  This file is the slow, index-order,
 * fp64 statement of what one speculative-decoding round of TABED computes.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  It shares no code, header, table or helper with the HIP library.
 *
 * What it follows (paper sections):
 *   - Sec. 3 "Preliminaries", items 1-3: draft gamma tokens, verify in
 *     parallel, accept token y with probability min(1, p(y)/q(y)); at the
 *     first rejection drop the rest and resample from norm(max(0, p - q)).
 *   - Sec. 5.1 "Proposed Method" + Algorithm 1: the m drafting methods run
 *     as one batch through the shared draft model; their distributions are
 *     mixed by a weighted average (W-Avg) and the next draft token is sampled
 *     from the mixture; the weights are chosen at the start of a block from
 *     the accumulated distance e_t^j = sum_{t'} D_KL(p_t' || q_t'^j) over the
 *     last h verified positions and held for the whole block.
 *   - App. B.2: the many-draft policy w = softmax([1/e^(1)..1/e^(m)]; tau),
 *     tau = 1, and the two-draft policy that scores the fixed candidates
 *     w^c = [1 - c/10, c/10] by the accumulated distance of the MIXTURE
 *     q(.; w^c) from the target and takes the arg-min (Alg. 1 (arg-min step));
 *     Sec. 5.1 last paragraph: TVD as the alternative distance; Sec. 5.1:
 *     selection by hard labels (token matches) instead of soft labels.
 *   - Eq. 1: speedup = block_eff / (gamma * Tq/Tp + 1).
 *   - Sec. 6.1, "Verification: Integrating Token Tree" (+ App. D): the drafts
 *     form a token tree of width 2 or 3 that the target verifies in one pass.
 *     The paper gives no construction; the one taken here is stated at
 *     oracle_draft_siblings / oracle_verify_tree.
 *
 * Notation: n = number of drafting methods (the paper's m), B independent
 * sequences, V vocabulary, d draft hidden size, gamma block length, h window.
 *
 * Where the paper is silent or ambiguous the reading taken is stated at the
 * function that takes it, marked "reading:".
 *
 * Pin status: every function below is pinned by tests that do not reuse its
 * formula: library cross-checks, closed forms, exact enumeration on tiny
 * vocabularies, the lossless-sampling invariant; oracle_philox4x32_10 is
 * compared word for word with rocRAND's Philox4x32-10 engine (another
 * author's implementation, compiled for the host from the library's public
 * header) on random 64-bit keys and 128-bit counters.
 *
 * All floating point is fp64 unless a value is an interface value that the
 * method stores in fp32 (logits, q(y), p(y), dev, ring, weights).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_FLAG_ACCEPT_MARGIN 1u /* accept test closer than 1e-6 relative   */
#define ORACLE_FLAG_SAMPLE_MARGIN 2u /* CDF edge / arg-max tie closer than 1e-6 */
#define ORACLE_FLAG_DEGENERATE    4u /* empty residual or CDF never crossed     */

static const double MARGIN = 1e-6;

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon et al., SC'11): counter-based generator.      */
/* ------------------------------------------------------------------ */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)M0 * c0;
        uint64_t p1 = (uint64_t)M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * reading: the uniforms of a round depend only on (seed, round, b, pos):
 * key = (seed lo, seed hi), counter = (round lo, round hi, b, pos).
 * For pos < gamma word 0 is the draft-sampling uniform and word 1 the
 * accept-test uniform; at pos = gamma word 0 drives the residual or bonus
 * sample.  u = (x >> 8) * 2^-24 lies in [0,1) and is exact in fp32.
 */
float oracle_uniform(uint64_t seed, uint64_t round, uint32_t b, uint32_t pos, int word)
{
    uint32_t ctr[4] = { (uint32_t)round, (uint32_t)(round >> 32), b, pos };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    return (float)(out[word & 3] >> 8) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------------------------ */
/* Eq. 1: expected walltime speedup from block efficiency.             */
/* ------------------------------------------------------------------ */
double oracle_speedup(double block_eff, double gamma, double tq_over_tp)
{
    return block_eff / (gamma * tq_over_tp + 1.0);
}

/* ------------------------------------------------------------------ */
/* LM head (Alg. 1 (draft forward), last layer of M_q): L[r,v] = sum_k H[r,k] W[v,k]. */
/* Storage values (fp32 or bf16) are upcast exactly; fp64 accumulation in    */
/* k order; one rounding to fp32 at the end.                                  */
/* ------------------------------------------------------------------ */
static double load_elem(const void* base, int dtype, size_t idx)
{
    if (dtype == 0) return (double)((const float*)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16; /* bf16 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

void oracle_lm_head(int M, int d, int V, int w_dtype, const void* W, const void* H, float* L)
{
    double* a = (double*)malloc((size_t)M * d * sizeof(double));
    for (size_t i = 0; i < (size_t)M * d; ++i) a[i] = load_elem(H, w_dtype, i);
#pragma omp parallel
    {
        double* wrow = (double*)malloc((size_t)d * sizeof(double));
#pragma omp for schedule(static)
        for (int v = 0; v < V; ++v) {
            for (int k = 0; k < d; ++k) wrow[k] = load_elem(W, w_dtype, (size_t)v * d + k);
            for (int r = 0; r < M; ++r) {
                double acc = 0.0;
                for (int k = 0; k < d; ++k) acc += a[(size_t)r * d + k] * wrow[k];
                L[(size_t)r * V + v] = (float)acc;
            }
        }
        free(wrow);
    }
    free(a);
}

/* ------------------------------------------------------------------ */
/* Vocabulary-wide building blocks.                                    */
/* ------------------------------------------------------------------ */

/* softmax of logits / T_eff; returns log-sum-exp of the scaled logits.
 * p and logp may be NULL. */
double oracle_softmax(const float* logits, int V, double T_eff, double* p, double* logp)
{
    double m = -INFINITY;
    for (int v = 0; v < V; ++v) {
        double s = (double)logits[v] / T_eff;
        if (s > m) m = s;
    }
    double Z = 0.0;
    for (int v = 0; v < V; ++v) Z += exp((double)logits[v] / T_eff - m);
    double lse = m + log(Z);
    for (int v = 0; v < V; ++v) {
        double lp = (double)logits[v] / T_eff - lse;
        if (logp) logp[v] = lp;
        if (p) p[v] = exp(lp);
    }
    return lse;
}

/* W-Avg (Alg. 1 (W-Avg step)): probability-space weighted average of n rows. */
void oracle_ensemble(int n, int V, const double* q, const float* w, double* q_ens)
{
    for (int v = 0; v < V; ++v) {
        double acc = 0.0;
        for (int j = 0; j < n; ++j) acc += (double)w[j] * q[(size_t)j * V + v];
        q_ens[v] = acc;
    }
}

/* reading: arg-max ties go to the lowest index; the decision is flagged when
 * the runner-up is within 1e-6 relative of the maximum. */
int oracle_argmax(const double* f, int V, uint32_t* flag)
{
    int best = 0;
    for (int v = 1; v < V; ++v) if (f[v] > f[best]) best = v;
    double second = -INFINITY;
    for (int v = 0; v < V; ++v) if (v != best && f[v] > second) second = f[v];
    if (flag && V > 1 && (f[best] - second) < MARGIN * fabs(f[best])) *flag |= ORACLE_FLAG_SAMPLE_MARGIN;
    return best;
}

static int argmax_logits(const float* x, int V)
{
    int best = 0;
    for (int v = 1; v < V; ++v) if (x[v] > x[best]) best = v;
    return best;
}

/* reading: Sample(f, u) is the inverse CDF of the (possibly unnormalised)
 * non-negative f: the smallest v whose inclusive prefix sum exceeds u * Z,
 * Z = sum f.  If rounding lets no prefix exceed it, the last v with f(v) > 0.
 * Flagged when u * Z lies within 1e-6 * Z of either edge of the chosen bin. */
int oracle_sample_cdf(const double* f, int V, double u, uint32_t* flag)
{
    double Z = 0.0;
    for (int v = 0; v < V; ++v) Z += f[v];
    double target = u * Z;
    double c = 0.0;
    for (int v = 0; v < V; ++v) {
        double prev = c;
        c += f[v];
        if (c > target) {
            if (flag) {
                if (fabs(c - target) < MARGIN * Z && v + 1 < V) *flag |= ORACLE_FLAG_SAMPLE_MARGIN;
                if (v > 0 && fabs(prev - target) < MARGIN * Z) *flag |= ORACLE_FLAG_SAMPLE_MARGIN;
            }
            return v;
        }
    }
    int last = V - 1;
    for (int v = V - 1; v >= 0; --v) if (f[v] > 0.0) { last = v; break; }
    if (flag) *flag |= ORACLE_FLAG_SAMPLE_MARGIN | ORACLE_FLAG_DEGENERATE;
    return last;
}

/* D_KL(p || q) = sum_v p(v) (log p(v) - log q(v)), from log-probabilities;
 * a term with p(v) == 0 contributes 0.  (Sec. 5.1, the formula for e_t^j.) */
double oracle_kl(const double* p, const double* logp, const double* logq, int V)
{
    double acc = 0.0;
    for (int v = 0; v < V; ++v) if (p[v] > 0.0) acc += p[v] * (logp[v] - logq[v]);
    return acc;
}

/* Total variation distance, the alternative D of Sec. 5.1. */
double oracle_tvd(const double* p, const double* q, int V)
{
    double acc = 0.0;
    for (int v = 0; v < V; ++v) acc += fabs(p[v] - q[v]);
    return 0.5 * acc;
}

/* ------------------------------------------------------------------ */
/* Alg. 1 (loop body: draft forward, W-Avg, Sample) for one in-block position, all B sequences.        */
/* ------------------------------------------------------------------ */
/* Layouts: W [V,d], H [B,n,d] (w_dtype 0 fp32 / 1 bf16), weights [B,n],
 * temperature [B] (0 => greedy row), u_draft [B,gamma] or NULL (=> Philox),
 * draft_logits [gamma,B,n,V], draft_lse [gamma,B,n] (fp64), draft_tokens
 * [B,gamma], draft_q [B,gamma], flags [B,gamma].
 * reading: a greedy row takes arg-max decisions but its distributions are the
 * untempered softmax (T_eff = 1), because the paper runs greedy decoding while
 * scoring drafts with soft-label KL. */
void oracle_draft_step(int V, int d, int n, int B, int gamma, int w_dtype,
                       uint64_t seed, uint64_t round, int pos,
                       const void* W, const void* H, const float* weights,
                       const float* temperature, const float* u_draft,
                       float* draft_logits, double* draft_lse, int32_t* draft_tokens,
                       float* draft_q, uint8_t* flags)
{
    float* L = draft_logits + (size_t)pos * B * n * V;
    oracle_lm_head(B * n, d, V, w_dtype, W, H, L);
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double T = (double)temperature[b];
        double T_eff = T > 0.0 ? T : 1.0;
        double* q = (double*)malloc((size_t)n * V * sizeof(double));
        double* q_ens = (double*)malloc((size_t)V * sizeof(double));
        for (int j = 0; j < n; ++j) {
            double lse = oracle_softmax(L + ((size_t)b * n + j) * V, V, T_eff, q + (size_t)j * V, NULL);
            draft_lse[((size_t)pos * B + b) * n + j] = lse;
        }
        oracle_ensemble(n, V, q, weights + (size_t)b * n, q_ens);
        uint32_t flag = 0;
        int y;
        if (T > 0.0) {
            float u = u_draft ? u_draft[(size_t)b * gamma + pos]
                              : oracle_uniform(seed, round, (uint32_t)b, (uint32_t)pos, 0);
            y = oracle_sample_cdf(q_ens, V, (double)u, &flag);
        } else {
            y = oracle_argmax(q_ens, V, &flag);
        }
        draft_tokens[(size_t)b * gamma + pos] = y;
        draft_q[(size_t)b * gamma + pos] = (float)q_ens[y];
        flags[(size_t)b * gamma + pos] = (uint8_t)flag;
        free(q); free(q_ens);
    }
}

/* ------------------------------------------------------------------ */
/* Sec. 3 items 2-3 + the per-position distances of Alg. 1 (arg-min step).     */
/* ------------------------------------------------------------------ */
/* target_logits [B,gamma+1,V]; u_acc [B,gamma] / u_res [B] or NULL (=> Philox).
 * Outputs: accept_len [B] = k; out_tokens [B,gamma+1] = the k accepted draft
 * tokens, then one corrected (k < gamma) or bonus (k = gamma) token, then -1;
 * dev [B,gamma,DW] for every i < gamma (meaningful for i < n_valid), where
 * with n_cand = 0: DW = n and dev[.,i,j] = D(p_i, q_i^(j)); with n_cand = 11
 * (n = 2): DW = 11 and dev[.,i,c] = D(p_i, (1 - c/10) q_i^(1) + (c/10) q_i^(2));
 * n_valid [B] = min(k+1, gamma); flags [B,gamma+1].
 * reading: the accept test is u * q(y) < p(y), evaluated in fp32 on the fp32
 * interface values; greedy rows accept iff y equals the arg-max of the target
 * logits, and emit that arg-max as corrected / bonus token.
 * reading: when all gamma tokens are accepted one bonus token is drawn from
 * p_gamma, so a round emits k+1 tokens.
 * reading: only positions 0..min(k, gamma-1) have both a verified target
 * distribution and draft distributions conditioned on kept tokens, hence
 * n_valid. */
#define ORACLE_GRID_CANDIDATES 11 /* c = 0..10, reading: both pure drafts are candidates */

/* Width of one distance vector: n per-draft distances, or 11 candidate mixtures (n_cand = 11, n = 2). */
int oracle_dev_width(int n, int n_cand) { return n_cand > 0 ? n_cand : n; }

void oracle_verify(int V, int n, int B, int gamma, int distance, int n_cand,
                   uint64_t seed, uint64_t round,
                   const float* target_logits, const float* draft_logits,
                   const int32_t* draft_tokens, const float* draft_q,
                   const float* weights, const float* temperature,
                   const float* u_acc, const float* u_res,
                   int32_t* accept_len, int32_t* out_tokens, float* dev,
                   int32_t* n_valid, uint8_t* flags)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double T = (double)temperature[b];
        int greedy = !(T > 0.0);
        double T_eff = greedy ? 1.0 : T;
        const float* Lt = target_logits + (size_t)b * (gamma + 1) * V;
        double* p = (double*)malloc((size_t)V * sizeof(double));
        double* logp = (double*)malloc((size_t)V * sizeof(double));
        double* q = (double*)malloc((size_t)n * V * sizeof(double));
        double* logq = (double*)malloc((size_t)n * V * sizeof(double));
        double* f = (double*)malloc((size_t)V * sizeof(double));
        double* mixlog = (double*)malloc((size_t)V * sizeof(double));
        uint8_t* fl = flags + (size_t)b * (gamma + 1);
        for (int i = 0; i <= gamma; ++i) fl[i] = 0;
        /* hard labels (distance 2): arg-max token of every candidate distribution at every position */
        int* pred = (int*)malloc((size_t)gamma * 64 * sizeof(int));
        /* reading: a mixture's arg-max whose runner-up is within the margin flags the position it labels (the
         * arg-max of a single draft is decided by its fp32 logits, the same on every implementation: no flag) */
        uint8_t* near_tie = (uint8_t*)calloc((size_t)gamma * 64, 1);

        int k = 0, rejected = 0;
        for (int i = 0; i < gamma; ++i) {
            oracle_softmax(Lt + (size_t)i * V, V, T_eff, p, logp);
            const int DW = oracle_dev_width(n, n_cand);
            for (int j = 0; j < n; ++j) {
                const float* Lq = draft_logits + (((size_t)i * B + b) * n + j) * V;
                oracle_softmax(Lq, V, T_eff, q + (size_t)j * V, logq + (size_t)j * V);
                if (n_cand > 0) continue;
                if (distance == 2) { pred[i * 64 + j] = oracle_argmax(q + (size_t)j * V, V, NULL); continue; }
                double D = distance == 0 ? oracle_kl(p, logp, logq + (size_t)j * V, V)
                                         : oracle_tvd(p, q + (size_t)j * V, V);
                dev[((size_t)b * gamma + i) * DW + j] = (float)D;
            }
            for (int c = 0; c < n_cand; ++c) { /* candidate mixtures of the two drafts */
                const double w1 = (double)c / (double)(n_cand - 1), w0 = 1.0 - w1;
                for (int v = 0; v < V; ++v) {
                    f[v] = w0 * q[v] + w1 * q[(size_t)V + v];
                    mixlog[v] = log(f[v]);
                }
                if (distance == 2) {
                    uint32_t tie = 0;
                    pred[i * 64 + c] = oracle_argmax(f, V, &tie);
                    near_tie[i * 64 + c] = tie ? 1 : 0;
                    continue;
                }
                double D = distance == 0 ? oracle_kl(p, logp, mixlog, V) : oracle_tvd(p, f, V);
                dev[((size_t)b * gamma + i) * DW + c] = (float)D;
            }
            if (rejected || k < i) continue; /* later positions: distances only */
            int y = draft_tokens[(size_t)b * gamma + i];
            int ok;
            if (greedy) {
                ok = (y == argmax_logits(Lt + (size_t)i * V, V));
            } else {
                float u = u_acc ? u_acc[(size_t)b * gamma + i]
                                : oracle_uniform(seed, round, (uint32_t)b, (uint32_t)i, 1);
                float qy = draft_q[(size_t)b * gamma + i];
                float py = (float)p[y];
                float lhs = u * qy;
                ok = lhs < py;
                double a = (double)lhs, c = (double)py;
                if (fabs(a - c) < MARGIN * fmax(a, c)) fl[i] |= ORACLE_FLAG_ACCEPT_MARGIN;
            }
            if (ok) { k++; continue; }
            rejected = 1;
            /* corrected token at the rejected position */
            int tok;
            if (greedy) {
                tok = argmax_logits(Lt + (size_t)i * V, V);
            } else {
                oracle_ensemble(n, V, q, weights + (size_t)b * n, f); /* f = q_ens,i */
                double Z = 0.0;
                for (int v = 0; v < V; ++v) { f[v] = fmax(0.0, p[v] - f[v]); Z += f[v]; }
                uint32_t flag = 0;
                float u = u_res ? u_res[b] : oracle_uniform(seed, round, (uint32_t)b, (uint32_t)gamma, 0);
                if (!(Z > 0.0)) { /* reading: empty residual => draw from p itself */
                    flag |= ORACLE_FLAG_DEGENERATE;
                    tok = oracle_sample_cdf(p, V, (double)u, &flag);
                } else {
                    tok = oracle_sample_cdf(f, V, (double)u, &flag);
                }
                fl[i] |= (uint8_t)flag;
            }
            out_tokens[(size_t)b * (gamma + 1) + i] = tok;
        }
        if (!rejected) { /* all gamma accepted: bonus token from p_gamma */
            int tok;
            if (greedy) {
                tok = argmax_logits(Lt + (size_t)gamma * V, V);
            } else {
                oracle_softmax(Lt + (size_t)gamma * V, V, T_eff, p, NULL);
                uint32_t flag = 0;
                float u = u_res ? u_res[b] : oracle_uniform(seed, round, (uint32_t)b, (uint32_t)gamma, 0);
                tok = oracle_sample_cdf(p, V, (double)u, &flag);
                fl[gamma] |= (uint8_t)flag;
            }
            out_tokens[(size_t)b * (gamma + 1) + gamma] = tok;
        }
        for (int i = 0; i < k; ++i)
            out_tokens[(size_t)b * (gamma + 1) + i] = draft_tokens[(size_t)b * gamma + i];
        for (int i = k + 1; i <= gamma; ++i) out_tokens[(size_t)b * (gamma + 1) + i] = -1;
        accept_len[b] = k;
        n_valid[b] = k + 1 < gamma ? k + 1 : gamma;
        if (distance == 2) {
            /* reading: the hard label of a verified position is the token emitted there (accepted draft token,
             * or the corrected token at the rejected position); "matches sampled from q^j" is taken as the
             * arg-max of the candidate distribution; the distance is the mismatch indicator, so that the
             * window sum counts mismatches and its arg-min maximises matches.  Positions beyond the rejected
             * one have no label: 1. */
            const int DW = oracle_dev_width(n, n_cand);
            for (int i = 0; i < gamma; ++i)
                for (int c = 0; c < DW; ++c) {
                    const int label = i <= k ? out_tokens[(size_t)b * (gamma + 1) + i] : -1;
                    dev[((size_t)b * gamma + i) * DW + c] = (pred[i * 64 + c] == label) ? 0.0f : 1.0f;
                    if (i <= k && near_tie[i * 64 + c]) fl[i] |= ORACLE_FLAG_SAMPLE_MARGIN;
                }
        }
        free(p); free(logp); free(q); free(logq); free(f); free(mixlog); free(pred); free(near_tie);
    }
}

/* ------------------------------------------------------------------ */
/* Alg. 1 (weight-selection step) with the App. B.2 many-draft policy.               */
/* ------------------------------------------------------------------ */
/* ring [B,h,n] holds the last <= h per-position distance vectors of each
 * sequence; ring_head [B] is the next slot to overwrite, ring_count [B] the
 * number of live slots.  dev / n_valid may be NULL (nothing to push).
 * policy 0: w = softmax((1 / max(e_j, eps)) / tau_w), e_j = sum over the
 * window; policy 1: equal weights; policy 2 (n = 2, window entries are the 11
 * candidate distances): w = [1 - c/10, c/10] for the candidate c with the
 * smallest window sum (reading: lowest c on ties; equal weights while the
 * window is empty); policy 3: the random-weights ablation of Sec. 6.2 (reading:
 * uniform on the simplex, drawn afresh for every block: w_j = E_j / sum E,
 * E_j = -ln U_j, U_j = (x + 0.5) 2^-24 from word j % 4 of the Philox block
 * (seed; round, b, gamma + 1 + j / 4), `round` being the block the weights are
 * for); the window is still maintained.  The window holds vectors of width DW = n (policies 0, 1)
 * or 11 (policy 2).
 * reading: an empty window gives equal weights; a window with fewer than h
 * entries sums what exists; 1/e is clamped by eps; softmax(x; tau) divides
 * by tau. */
void oracle_update_weights(int n, int B, int gamma, int h, int policy,
                           double tau_w, double eps, uint64_t seed, uint64_t round,
                           const float* dev, const int32_t* n_valid,
                           float* ring, int32_t* ring_head, int32_t* ring_count,
                           float* weights)
{
    const int DW = policy == 2 ? ORACLE_GRID_CANDIDATES : n;
    const int all = (h == 0);
    if (all) h = 1;
    for (int b = 0; b < B; ++b) {
        if (dev && n_valid) {
            for (int i = 0; i < n_valid[b]; ++i) {
                if (all) { /* running sum, one fp32 addition per verified position, in order */
                    for (int j = 0; j < DW; ++j)
                        ring[(size_t)b * DW + j] = ring[(size_t)b * DW + j] + dev[((size_t)b * gamma + i) * DW + j];
                    if (ring_count[b] < INT32_MAX) ring_count[b]++;
                    continue;
                }
                int slot = ring_head[b];
                for (int j = 0; j < DW; ++j)
                    ring[((size_t)b * h + slot) * DW + j] = dev[((size_t)b * gamma + i) * DW + j];
                ring_head[b] = (slot + 1) % h;
                if (ring_count[b] < h) ring_count[b]++;
            }
        }
        float* w = weights + (size_t)b * n;
        int count = ring_count[b];
        if (all && count > 1) count = 1; /* the single slot already holds the sum; head stays 0 */
        if (policy == 3) {
            double E[64], tot = 0.0;
            for (int j = 0; j < n; ++j) {
                uint32_t ctr[4] = { (uint32_t)round, (uint32_t)(round >> 32), (uint32_t)b, (uint32_t)(gamma + 1 + j / 4) };
                uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
                uint32_t out[4];
                oracle_philox4x32_10(ctr, key, out);
                E[j] = -log(((double)(out[j % 4] >> 8) + 0.5) * (1.0 / 16777216.0));
                tot += E[j];
            }
            for (int j = 0; j < n; ++j) w[j] = (float)(E[j] / tot);
            continue;
        }
        if (policy == 1 || count == 0) {
            for (int j = 0; j < n; ++j) w[j] = (float)(1.0 / n);
            continue;
        }
        double x[64];
        double xmax = -INFINITY;
        if (policy == 2) { /* arg-min over the candidate mixtures */
            int best = 0;
            double ebest = INFINITY;
            for (int c = 0; c < DW; ++c) {
                double e = 0.0;
                for (int t = 0; t < count; ++t) {
                    int slot = ((ring_head[b] - count + t) % h + h) % h;
                    e += (double)ring[((size_t)b * h + slot) * DW + c];
                }
                if (e < ebest) { ebest = e; best = c; }
            }
            const double w1 = (double)best / (double)(DW - 1);
            w[0] = (float)(1.0 - w1);
            w[1] = (float)w1;
            continue;
        }
        for (int j = 0; j < n; ++j) {
            double e = 0.0;
            for (int t = 0; t < count; ++t) { /* oldest .. newest */
                int slot = ((ring_head[b] - count + t) % h + h) % h;
                e += (double)ring[((size_t)b * h + slot) * n + j];
            }
            x[j] = (1.0 / fmax(e, eps)) / tau_w;
            if (x[j] > xmax) xmax = x[j];
        }
        double Z = 0.0;
        for (int j = 0; j < n; ++j) Z += exp(x[j] - xmax);
        for (int j = 0; j < n; ++j) w[j] = (float)(exp(x[j] - xmax) / Z);
    }
}

/* ------------------------------------------------------------------ */
/* Token tree (Sec. 6.1 "Verification: Integrating Token Tree").        */
/* ------------------------------------------------------------------ */
/*
 * reading (the paper names the tree width, 2 or 3, and nothing else): at every
 * in-block position i the draft proposes `width` sibling candidates for the
 * same prefix, all taken from the ensembled distribution q_i of that position:
 * candidate 0 is the token Alg. 1 (Sample step) samples (the "trunk": the only one
 * the draft model extends to position i+1), candidates 1..width-1 are leaves.
 * A sampling row draws the siblings independently from q_i (inverse CDF, own
 * uniform each); a greedy row takes the next-largest entries of q_i (lowest
 * index on ties), so its candidates are the top `width` tokens in order.
 * Width 1 is the plain chain.
 *
 * Sibling s (1-based) of position pos uses the Philox block of counter
 * (round, b, pos + s * 65536): word 0 draws the sibling, word 1 is its accept
 * uniform.
 *
 * Layouts: draft_logits [gamma,B,n,V] (slot pos already written by
 * oracle_draft_step), draft_tokens [B,gamma] (trunk tokens, column pos
 * written), u_sib [B,gamma,width-1] or NULL; outputs sib_tokens, sib_q,
 * sib_flags [B,gamma,width-1], entries (b,pos,.) written.
 */
#define ORACLE_SIB_STRIDE 65536u

void oracle_draft_siblings(int V, int n, int B, int gamma, int width,
                           uint64_t seed, uint64_t round, int pos,
                           const float* draft_logits, const int32_t* draft_tokens,
                           const float* weights, const float* temperature, const float* u_sib,
                           int32_t* sib_tokens, float* sib_q, uint8_t* sib_flags)
{
    const int S = width - 1;
    if (S <= 0) return;
    const float* L = draft_logits + (size_t)pos * B * n * V;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double T = (double)temperature[b];
        double T_eff = T > 0.0 ? T : 1.0;
        double* q = (double*)malloc((size_t)n * V * sizeof(double));
        double* q_ens = (double*)malloc((size_t)V * sizeof(double));
        double* rest = (double*)malloc((size_t)V * sizeof(double));
        for (int j = 0; j < n; ++j) oracle_softmax(L + ((size_t)b * n + j) * V, V, T_eff, q + (size_t)j * V, NULL);
        oracle_ensemble(n, V, q, weights + (size_t)b * n, q_ens);
        for (int v = 0; v < V; ++v) rest[v] = q_ens[v];
        int trunk = draft_tokens[(size_t)b * gamma + pos];
        if (trunk >= 0 && trunk < V) rest[trunk] = -1.0; /* greedy rows: already taken */
        for (int s = 1; s <= S; ++s) {
            size_t o = ((size_t)b * gamma + pos) * S + (s - 1);
            uint32_t flag = 0;
            int y;
            if (T > 0.0) {
                float u = u_sib ? u_sib[o] : oracle_uniform(seed, round, (uint32_t)b, (uint32_t)pos + (uint32_t)s * ORACLE_SIB_STRIDE, 0);
                y = oracle_sample_cdf(q_ens, V, (double)u, &flag);
            } else {
                y = oracle_argmax(rest, V, &flag);  /* next-largest entry; -1 marks the ones already taken */
                rest[y] = -1.0;
            }
            sib_tokens[o] = y;
            sib_q[o] = (float)q_ens[y];
            sib_flags[o] = (uint8_t)flag;
        }
        free(q); free(q_ens); free(rest);
    }
}

/*
 * Verification of the tree (reading, continued).  The walk goes down the trunk
 * exactly as the chain does (same test, same uniforms) until the trunk token of
 * some position k is rejected, or all gamma are accepted (bonus token from
 * p_gamma, as in the chain).  At position k the siblings are tried in order by
 * multi-round rejection sampling, the lossless rule for several candidates
 * drawn from one proposal: with f_0 = p_k, Z_0 = 1 and, after each rejection,
 *     f_c(v) = max(0, f_{c-1}(v) / Z_{c-1} - q_k(v)),   Z_c = sum_v f_c(v),
 * candidate c (c >= 1) is accepted iff  u_c * q_k(y_c) * Z_c < f_c(y_c)
 * (probability min(1, r_c(y)/q(y)) with r_c = f_c / Z_c; c = 0 is the chain's
 * own test u * q < p).  An accepted sibling is emitted and, being a leaf, is
 * followed by one bonus token from the target's distribution AFTER it
 * (leaf_logits); if every candidate is rejected the corrected token comes from
 * r_width = f_width / Z_width.  The one final draw of a round (corrected token,
 * bonus after a leaf, or bonus after gamma accepts) uses the chain's u_res.
 * Greedy rows: a candidate is accepted iff it equals arg-max p_k; the bonus
 * after a leaf is the arg-max of its leaf row; otherwise arg-max p_k is emitted.
 * The decision of a sibling test is taken in fp64 on the fp32 interface value
 * q(y); it is flagged when |lhs - rhs| < 1e-6 * max(f_{c-1}(y)/Z_{c-1}, q(y)).
 * An empty residual (Z_c = 0) ends the levels: the token is drawn from p_k,
 * flagged degenerate.
 * The distances and n_valid = min(k+1, gamma) are those of the chain: the
 * position where the walk ends is verified either way.
 *
 * Extra inputs: leaf_logits [B,gamma,width-1,V] (target logits after sibling
 * s of position i), sib_tokens / sib_q [B,gamma,width-1], u_acc_sib
 * [B,gamma,width-1] or NULL.  Extra outputs: leaf [B] = 0 or the 1-based index
 * of the accepted sibling; n_out [B] = emitted tokens (k+1, or k+2 after a
 * leaf); out_tokens [B,gamma+1] as in oracle_verify with the leaf and its bonus
 * token at columns k and k+1; flags [B,gamma+1]: column k also carries the
 * sibling tests' margin bits, column k+1 the bonus draw after a leaf.
 */
void oracle_verify_tree(int V, int n, int B, int gamma, int width, int distance,
                        uint64_t seed, uint64_t round,
                        const float* target_logits, const float* leaf_logits,
                        const float* draft_logits,
                        const int32_t* draft_tokens, const float* draft_q,
                        const int32_t* sib_tokens, const float* sib_q,
                        const float* weights, const float* temperature,
                        const float* u_acc, const float* u_res, const float* u_acc_sib,
                        int32_t* accept_len, int32_t* out_tokens, float* dev,
                        int32_t* n_valid, uint8_t* flags, int32_t* leaf, int32_t* n_out)
{
    /* the trunk: everything the chain computes */
    oracle_verify(V, n, B, gamma, distance, 0, seed, round, target_logits, draft_logits, draft_tokens, draft_q,
                  weights, temperature, u_acc, u_res, accept_len, out_tokens, dev, n_valid, flags);
    const int S = width - 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int k = accept_len[b];
        leaf[b] = 0;
        n_out[b] = k + 1;
        if (S <= 0 || k >= gamma) continue;
        double T = (double)temperature[b];
        int greedy = !(T > 0.0);
        double T_eff = greedy ? 1.0 : T;
        const float* Lt = target_logits + ((size_t)b * (gamma + 1) + k) * V;
        uint8_t* fl = flags + (size_t)b * (gamma + 1);
        int32_t* out = out_tokens + (size_t)b * (gamma + 1);
        double* f = (double*)malloc((size_t)V * sizeof(double));
        double* q = (double*)malloc((size_t)n * V * sizeof(double));
        double* q_ens = (double*)malloc((size_t)V * sizeof(double));
        double* p = (double*)malloc((size_t)V * sizeof(double));
        int accepted = 0;
        if (greedy) {
            int top = argmax_logits(Lt, V);
            for (int s = 1; s <= S && !accepted; ++s)
                if (sib_tokens[((size_t)b * gamma + k) * S + (s - 1)] == top) accepted = s;
            if (accepted) {
                out[k] = top;
                out[k + 1] = argmax_logits(leaf_logits + (((size_t)b * gamma + k) * S + (accepted - 1)) * V, V);
            }
        } else {
            oracle_softmax(Lt, V, T_eff, p, NULL);
            for (int j = 0; j < n; ++j)
                oracle_softmax(draft_logits + (((size_t)k * B + b) * n + j) * V, V, T_eff, q + (size_t)j * V, NULL);
            oracle_ensemble(n, V, q, weights + (size_t)b * n, q_ens);
            for (int v = 0; v < V; ++v) f[v] = p[v];
            double Zprev = 1.0;
            uint32_t flag = 0;
            int degenerate = 0;
            for (int c = 1; c <= width; ++c) {
                /* candidate c-1 was rejected: f_c = max(0, f_{c-1}/Z_{c-1} - q); sibling c, if there is one, is
                 * tested against it, otherwise (c = width) the corrected token is drawn from it */
                int y = -1;
                double qy = 0.0, minuend_y = 0.0;
                if (c <= S) {
                    y = sib_tokens[((size_t)b * gamma + k) * S + (c - 1)];
                    qy = (double)sib_q[((size_t)b * gamma + k) * S + (c - 1)];
                    minuend_y = (y >= 0 && y < V) ? f[y] / Zprev : 0.0;   /* f_{c-1}(y) / Z_{c-1}, kept for the margin */
                }
                double Z = 0.0;
                for (int v = 0; v < V; ++v) { f[v] = fmax(0.0, f[v] / Zprev - q_ens[v]); Z += f[v]; }
                if (!(Z > 0.0)) { degenerate = 1; break; }
                Zprev = Z;
                if (c > S) break;                            /* every candidate rejected: f = f_width */
                if (y < 0 || y >= V) { flag |= ORACLE_FLAG_DEGENERATE; continue; }
                float u = u_acc_sib ? u_acc_sib[((size_t)b * gamma + k) * S + (c - 1)]
                                    : oracle_uniform(seed, round, (uint32_t)b, (uint32_t)k + (uint32_t)c * ORACLE_SIB_STRIDE, 1);
                double fy = fmax(0.0, minuend_y - qy);      /* f_c(y) on the interface value q(y) */
                double lhs = (double)u * qy * Z;
                if (fabs(lhs - fy) < MARGIN * fmax(minuend_y, qy)) flag |= ORACLE_FLAG_ACCEPT_MARGIN;
                if (lhs < fy) { accepted = c; break; }
            }
            float u = u_res ? u_res[b] : oracle_uniform(seed, round, (uint32_t)b, (uint32_t)gamma, 0);
            fl[k] &= (uint8_t)~(ORACLE_FLAG_SAMPLE_MARGIN | ORACLE_FLAG_DEGENERATE);   /* the chain's draw is replaced */
            if (accepted) {
                out[k] = sib_tokens[((size_t)b * gamma + k) * S + (accepted - 1)];
                uint32_t bflag = 0;
                oracle_softmax(leaf_logits + (((size_t)b * gamma + k) * S + (accepted - 1)) * V, V, T_eff, p, NULL);
                out[k + 1] = oracle_sample_cdf(p, V, (double)u, &bflag);
                fl[k + 1] = (uint8_t)bflag;
            } else if (degenerate) {
                flag |= ORACLE_FLAG_DEGENERATE;
                out[k] = oracle_sample_cdf(p, V, (double)u, &flag);
            } else {
                out[k] = oracle_sample_cdf(f, V, (double)u, &flag);   /* f = f_width */
            }
            fl[k] |= (uint8_t)flag;
        }
        if (accepted) { leaf[b] = accepted; n_out[b] = k + 2; }
        free(f); free(q); free(q_ens); free(p);
    }
}
