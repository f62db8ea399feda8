"""Pins for the oracle's draft / verify / weight-update calls.

The core pin is exactness of speculative sampling: on tiny vocabularies the joint distribution of
(accepted length, emitted tokens) is computed here by brute-force enumeration of every draft token and
every accept/reject outcome, from nothing but the accept rule min(1, p/q) and the residual
norm(max(0, p-q)) of Sec. 3; the oracle -- driven either by a midpoint grid of uniforms or by its own
Philox uniforms -- must reproduce it, and its first emitted token must follow the target distribution
p_0 exactly (speculative decoding is lossless).
"""
import itertools

import numpy as np
import scipy.special as sp
import scipy.stats as st


def _identity_head(V):
    """fp32 W = I_V, so the 'hidden state' of a draft IS its logit row (a special case of the LM head)."""
    return np.eye(V, dtype=np.float32)


def _run_round(oracle, *, logq, logp, w, temperature, B, seed=0, rnd=0, u_draft=None, u_acc=None, u_res=None):
    """One SD round on B copies of the same distributions.  logq [gamma,n,V], logp [gamma+1,V]."""
    gamma, n, V = logq.shape
    W = _identity_head(V)
    dl = np.zeros((gamma, B, n, V), np.float32)
    lse = np.zeros((gamma, B, n), np.float64)
    tok = np.zeros((B, gamma), np.int32)
    dq = np.zeros((B, gamma), np.float32)
    fl = np.zeros((B, gamma), np.uint8)
    weights = np.tile(np.asarray(w, np.float32), (B, 1))
    temp = np.full(B, temperature, np.float32)
    for pos in range(gamma):
        H = np.ascontiguousarray(np.broadcast_to(logq[pos].astype(np.float32), (B, n, V)))
        oracle.draft_step(V=V, d=V, n=n, B=B, gamma=gamma, w_dtype=0, seed=seed, rnd=rnd, pos=pos, W=W, H=H,
                          weights=weights, temperature=temp, draft_logits=dl, draft_lse=lse, draft_tokens=tok,
                          draft_q=dq, flags=fl, u_draft=u_draft)
    tl = np.ascontiguousarray(np.broadcast_to(logp.astype(np.float32), (B, gamma + 1, V)))
    out = oracle.verify(V=V, n=n, B=B, gamma=gamma, distance=0, seed=seed, rnd=rnd, target_logits=tl,
                        draft_logits=dl, draft_tokens=tok, draft_q=dq, weights=weights, temperature=temp,
                        u_acc=u_acc, u_res=u_res)
    out.update(draft_tokens=tok, draft_q=dq, draft_logits=dl, draft_lse=lse, draft_flags=fl)
    return out


def _exact_joint(p, q):
    """Brute force over every draft sequence and accept pattern.  p [gamma+1,V], q [gamma,V] (the mixture).
    Returns {(k, emitted tokens...): probability} (positions are independent in the synthetic workload)."""
    gamma, V = q.shape
    joint = {}
    for k in range(gamma + 1):
        for ys in itertools.product(range(V), repeat=k):
            pref = 1.0
            for i, y in enumerate(ys):
                pref *= q[i, y] * min(1.0, p[i, y] / q[i, y])
            if pref == 0.0:
                continue
            if k == gamma:
                for z in range(V):
                    joint[(k,) + ys + (z,)] = pref * p[gamma, z]
            else:
                rej = sum(q[k, y] * (1.0 - min(1.0, p[k, y] / q[k, y])) for y in range(V))
                res = np.maximum(0.0, p[k] - q[k])
                if rej > 0:
                    for z in range(V):
                        if res[z] > 0:
                            joint[(k,) + ys + (z,)] = pref * rej * res[z] / res.sum()
    assert abs(sum(joint.values()) - 1.0) < 1e-6      # fp32 weights need not sum to 1 exactly
    return joint


def _dists(rng, gamma, n, V, w):
    logq = rng.standard_normal((gamma, n, V)) * 1.5
    logp = rng.standard_normal((gamma + 1, V)) * 1.5
    # library softmax on the fp32-rounded logits the oracle will see
    qj = sp.softmax(logq.astype(np.float32).astype(np.float64), axis=-1)
    p = sp.softmax(logp.astype(np.float32).astype(np.float64), axis=-1)
    q = np.tensordot(np.asarray(w, np.float32).astype(np.float64), qj, axes=([0], [1]))
    return logq, logp, p, q, qj


def _observed(out, gamma):
    seqs = {}
    for k, row in zip(out["accept_len"], out["out_tokens"]):
        key = (int(k),) + tuple(int(t) for t in row[: k + 1])
        assert all(t == -1 for t in row[k + 1:])
        seqs[key] = seqs.get(key, 0) + 1
    return seqs


def test_gamma1_uniform_grid_reproduces_exact_joint_and_is_lossless(oracle):
    rng = np.random.default_rng(11)
    V, n, gamma, w = 5, 2, 1, (0.3, 0.7)
    logq, logp, p, q, _ = _dists(rng, gamma, n, V, w)
    N = 48
    mid = (np.arange(N) + 0.5) / N
    ud, ua, ur = [a.ravel() for a in np.meshgrid(mid, mid, mid, indexing="ij")]
    B = N ** 3
    out = _run_round(oracle, logq=logq, logp=logp, w=w, temperature=1.0, B=B,
                     u_draft=ud.reshape(B, 1), u_acc=ua.reshape(B, 1), u_res=ur)
    exact = _exact_joint(p, q)
    obs = _observed(out, gamma)
    assert set(obs) <= set(exact)
    for key, pr in exact.items():
        assert abs(obs.get(key, 0) / B - pr) < 3.0 / N, key
    # lossless: the first emitted token follows p_0 whatever the draft mixture is
    first = np.bincount(out["out_tokens"][:, 0], minlength=V) / B
    np.testing.assert_allclose(first, p[0], atol=3.0 / N)
    # accepted-length law: P(k=1) = sum_v min(p, q)
    assert abs(np.mean(out["accept_len"] == 1) - np.minimum(p[0], q[0]).sum()) < 3.0 / N
    # interface values are what they claim to be
    np.testing.assert_allclose(out["draft_q"][:, 0], q[0][out["draft_tokens"][:, 0]], rtol=1e-6)


def test_gamma3_philox_rounds_match_enumeration_chi_square(oracle):
    rng = np.random.default_rng(12)
    V, n, gamma, w = 4, 3, 3, (0.5, 0.2, 0.3)
    logq, logp, p, q, _ = _dists(rng, gamma, n, V, w)
    B = 200_000
    out = _run_round(oracle, logq=logq, logp=logp, w=w, temperature=1.0, B=B, seed=0, rnd=5)
    exact = _exact_joint(p, q)
    obs = _observed(out, gamma)
    assert set(obs) <= set(exact)
    keys = sorted(exact)
    f_obs = np.array([obs.get(k, 0) for k in keys], float)
    f_exp = np.array([exact[k] for k in keys]) * B
    keep = f_exp >= 5
    chi = ((f_obs[keep] - f_exp[keep]) ** 2 / f_exp[keep]).sum() + \
        (f_obs[~keep].sum() - f_exp[~keep].sum()) ** 2 / max(f_exp[~keep].sum(), 1e-9)
    assert st.chi2.sf(chi, keep.sum()) > 1e-4
    # closed form of the accepted-length law with alpha_i = sum_v min(p_i, q_i)
    alpha = np.minimum(p[:gamma], q).sum(axis=1)
    law = [np.prod(alpha[:j]) * (1 - alpha[j]) for j in range(gamma)] + [np.prod(alpha)]
    cnt = np.bincount(out["accept_len"], minlength=gamma + 1)
    assert st.chisquare(cnt, np.array(law) * B).pvalue > 1e-4
    assert np.array_equal(out["n_valid"], np.minimum(out["accept_len"] + 1, gamma))
    # lossless at every depth: given that position i is reached with all earlier drafts accepted,
    # the token emitted there follows p_i
    for i in range(gamma + 1):
        sel = out["accept_len"] >= i
        emitted = out["out_tokens"][sel, i]
        assert st.chisquare(np.bincount(emitted, minlength=V), p[i] * sel.sum()).pvalue > 1e-4
    # block efficiency statistic: E[tokens] = 1 + sum_j prod_{i<j} alpha_i
    e_tok = 1 + sum(np.prod(alpha[:j]) for j in range(1, gamma + 1))
    assert abs((out["accept_len"] + 1).mean() - e_tok) < 5 * np.sqrt(gamma ** 2 / B)


def test_single_draft_reduces_to_textbook_speculative_sampling(oracle):
    """n = 1, w = [1]: accept probability of token y is min(1, p(y)/q(y)) exactly."""
    rng = np.random.default_rng(13)
    V = 6
    logq, logp, p, q, _ = _dists(rng, 1, 1, V, (1.0,))
    N = 2048
    mid = (np.arange(N) + 0.5) / N
    for y in range(V):
        # force draft token y: put the draft uniform in the middle of y's CDF bin
        cdf = np.concatenate([[0], np.cumsum(q[0])])
        ud = np.full((N, 1), (cdf[y] + cdf[y + 1]) / 2 / cdf[-1])
        out = _run_round(oracle, logq=logq, logp=logp, w=(1.0,), temperature=1.0, B=N,
                         u_draft=ud, u_acc=mid.reshape(N, 1), u_res=np.full(N, 0.5))
        assert np.all(out["draft_tokens"] == y)
        assert abs(np.mean(out["accept_len"]) - min(1.0, p[0, y] / q[0, y])) <= 1.0 / N
    # identical draft and target: always accepted
    out = _run_round(oracle, logq=logp[None, :1], logp=logp, w=(1.0,), temperature=1.0, B=4096, rnd=3)
    assert np.all(out["accept_len"] == 1)


def test_residual_is_max_p_minus_q_normalised(oracle):
    rng = np.random.default_rng(14)
    V = 6
    logq, logp, p, q, _ = _dists(rng, 1, 2, V, (0.4, 0.6))
    res = np.maximum(0, p[0] - q[0]); res /= res.sum()
    N = 4096
    mid = (np.arange(N) + 0.5) / N
    # u_acc just below 1 rejects every token with p<q; pick such a token as the draft
    y = int(np.argmax(q[0] - p[0]))
    cdf = np.concatenate([[0], np.cumsum(q[0])])
    out = _run_round(oracle, logq=logq, logp=logp, w=(0.4, 0.6), temperature=1.0, B=N,
                     u_draft=np.full((N, 1), (cdf[y] + cdf[y + 1]) / 2 / cdf[-1]),
                     u_acc=np.full((N, 1), 1 - 2.0 ** -24), u_res=mid)
    assert np.all(out["accept_len"] == 0)
    freq = np.bincount(out["out_tokens"][:, 0], minlength=V) / N
    np.testing.assert_allclose(freq, res, atol=1.5 / N)
    assert np.all(freq[p[0] <= q[0]] == 0)          # tokens with p<=q never come out of the residual


def test_greedy_round_matches_a_five_line_reference(oracle):
    rng = np.random.default_rng(15)
    V, n, gamma = 50, 3, 4
    for trial in range(40):
        w = rng.dirichlet(np.ones(n)).astype(np.float32)
        logq, logp, p, q, _ = _dists(rng, gamma, n, V, w)
        if trial % 2:                                # make the target agree with the draft on a prefix
            for i in range(trial % gamma + 1):
                logp[i, int(np.argmax(q[i]))] = logp[i].max() + 1
        out = _run_round(oracle, logq=logq, logp=logp, w=w, temperature=0.0, B=1)
        y = [int(np.argmax(q[i])) for i in range(gamma)]
        t = [int(np.argmax(logp[i].astype(np.float32))) for i in range(gamma + 1)]
        k = next((i for i in range(gamma) if y[i] != t[i]), gamma)
        ref = y[:k] + [t[k]] + [-1] * (gamma - k)
        assert out["draft_tokens"][0].tolist() == y
        assert out["accept_len"][0] == k and out["out_tokens"][0].tolist() == ref


def test_deviations_match_library_relative_entropy(oracle):
    rng = np.random.default_rng(16)
    V, n, gamma, w = 200, 3, 2, (0.2, 0.3, 0.5)
    logq, logp, p, q, qj = _dists(rng, gamma, n, V, w)
    for T in (1.0, 0.7):
        out = _run_round(oracle, logq=logq, logp=logp, w=w, temperature=T, B=2, rnd=1)
        pT = sp.softmax(logp.astype(np.float32).astype(np.float64) / T, axis=-1)
        qT = sp.softmax(logq.astype(np.float32).astype(np.float64) / T, axis=-1)
        for i in range(gamma):
            for j in range(n):
                ref = sp.rel_entr(pT[i], qT[i, j]).sum()            # KL(p || q_j), this direction
                assert abs(out["dev"][0, i, j] - ref) < 1e-6 * max(1, ref)
    # greedy rows score drafts with the untempered softmax (T_eff = 1)
    out = _run_round(oracle, logq=logq, logp=logp, w=w, temperature=0.0, B=1)
    assert abs(out["dev"][0, 1, 2] - sp.rel_entr(p[1], qj[1, 2]).sum()) < 1e-6


def test_tvd_distance_option(oracle):
    rng = np.random.default_rng(17)
    V, n, gamma = 30, 2, 2
    logq, logp, p, q, qj = _dists(rng, gamma, n, V, (0.5, 0.5))
    W = _identity_head(V)
    dl = np.ascontiguousarray(logq.astype(np.float32)[:, None])      # [gamma,1,n,V]
    out = oracle.verify(V=V, n=n, B=1, gamma=gamma, distance=1, seed=0, rnd=0,
                        target_logits=logp.astype(np.float32)[None], draft_logits=dl,
                        draft_tokens=np.zeros((1, gamma), np.int32), draft_q=np.ones((1, gamma), np.float32),
                        weights=np.full((1, n), 0.5, np.float32), temperature=np.ones(1, np.float32))
    for i in range(gamma):
        for j in range(n):
            assert abs(out["dev"][0, i, j] - 0.5 * np.abs(p[i] - qj[i, j]).sum()) < 1e-6


# ------------------------------------------------------------------ weights (Alg. 1 (weight-selection step), App. B.2)
def _fresh_ring(B, h, n):
    return np.zeros((B, h, n), np.float32), np.zeros(B, np.int32), np.zeros(B, np.int32)


def test_weights_empty_window_equal_and_static_policy(oracle):
    ring, head, count = _fresh_ring(3, 4, 5)
    w = oracle.update_weights(n=5, B=3, gamma=2, h=4, policy=0, tau_w=1.0, eps=1e-6, dev=None, n_valid=None,
                              ring=ring, ring_head=head, ring_count=count)
    assert np.all(w == np.float32(0.2))
    dev = np.random.default_rng(1).random((3, 2, 5)).astype(np.float32)
    w = oracle.update_weights(n=5, B=3, gamma=2, h=4, policy=1, tau_w=1.0, eps=1e-6, dev=dev,
                              n_valid=np.array([2, 1, 2], np.int32), ring=ring, ring_head=head, ring_count=count)
    assert np.all(w == np.float32(0.2)) and count.tolist() == [2, 1, 2]


def test_weights_two_draft_closed_form_and_simplex(oracle):
    rng = np.random.default_rng(21)
    for tau in (1.0, 0.5, 3.0):
        ring, head, count = _fresh_ring(1, 8, 2)
        dev = rng.random((1, 3, 2)).astype(np.float32) + 0.05
        w = oracle.update_weights(n=2, B=1, gamma=3, h=8, policy=0, tau_w=tau, eps=1e-6, dev=dev,
                                  n_valid=np.array([3], np.int32), ring=ring, ring_head=head, ring_count=count)
        e = dev[0].astype(np.float64).sum(axis=0)
        sig = 1.0 / (1.0 + np.exp(-((1 / e[0] - 1 / e[1]) / tau)))   # softmax over two = logistic
        assert abs(w[0, 0] - sig) < 1e-6 and abs(w.sum() - 1) < 1e-6 and np.all(w >= 0)
        assert (w[0, 0] > w[0, 1]) == (e[0] < e[1])                  # smaller error => larger weight
    # equal errors => uniform; zero error is clamped and takes (almost) everything
    ring, head, count = _fresh_ring(1, 4, 3)
    w = oracle.update_weights(n=3, B=1, gamma=1, h=4, policy=0, tau_w=1.0, eps=1e-6,
                              dev=np.full((1, 1, 3), 0.25, np.float32), n_valid=np.array([1], np.int32),
                              ring=ring, ring_head=head, ring_count=count)
    np.testing.assert_allclose(w, 1 / 3, rtol=1e-6)
    ring, head, count = _fresh_ring(1, 4, 3)
    w = oracle.update_weights(n=3, B=1, gamma=1, h=4, policy=0, tau_w=1.0, eps=1e-6,
                              dev=np.array([[[0.0, 0.0, 0.5]]], np.float32), n_valid=np.array([1], np.int32),
                              ring=ring, ring_head=head, ring_count=count)
    np.testing.assert_allclose(w[0], [0.5, 0.5, 0.0], atol=1e-6)


def test_window_is_the_last_h_valid_positions(oracle):
    """The ring must equal a brute-force recomputation from the full log of pushed positions."""
    rng = np.random.default_rng(22)
    B, n, gamma, h = 3, 4, 5, 7
    ring, head, count = _fresh_ring(B, h, n)
    log = [[] for _ in range(B)]
    for r in range(30):
        dev = (rng.random((B, gamma, n)) + 0.01).astype(np.float32)
        nv = rng.integers(1, gamma + 1, B).astype(np.int32)
        w = oracle.update_weights(n=n, B=B, gamma=gamma, h=h, policy=0, tau_w=1.0, eps=1e-6, dev=dev, n_valid=nv,
                                  ring=ring, ring_head=head, ring_count=count)
        for b in range(B):
            log[b] += [dev[b, i] for i in range(nv[b])]               # positions beyond n_valid never enter
            e = np.sum(np.asarray(log[b][-h:], np.float64), axis=0)
            np.testing.assert_allclose(w[b], sp.softmax(1.0 / e), rtol=2e-6)
            assert count[b] == min(len(log[b]), h) and head[b] == len(log[b]) % h


def test_weights_follow_the_draft_that_matches_the_target(oracle):
    """Adaptive behaviour: when the target switches to agree with another draft, the largest weight
    follows within a window's worth of verified positions."""
    rng = np.random.default_rng(23)
    V, n, gamma, h, B = 64, 3, 3, 6, 2
    W = _identity_head(V)
    ring, head, count = _fresh_ring(B, h, n)
    dev = nv = None
    lag = 0
    for rnd in range(60):
        jstar = (rnd // 20) % n
        w = oracle.update_weights(n=n, B=B, gamma=gamma, h=h, policy=0, tau_w=1.0, eps=1e-6, dev=dev, n_valid=nv,
                                  ring=ring, ring_head=head, ring_count=count)
        if rnd % 20 >= 8:
            assert np.all(np.argmax(w, axis=1) == jstar), (rnd, w)
        logq = rng.standard_normal((gamma + 1, B, n, V)).astype(np.float32) * 2
        tl = np.ascontiguousarray(np.transpose(logq[:, :, jstar], (1, 0, 2))) + \
            rng.standard_normal((B, gamma + 1, V)).astype(np.float32) * 0.3
        dl = np.zeros((gamma, B, n, V), np.float32); lse = np.zeros((gamma, B, n)); tok = np.zeros((B, gamma), np.int32)
        dq = np.zeros((B, gamma), np.float32); fl = np.zeros((B, gamma), np.uint8)
        for pos in range(gamma):
            oracle.draft_step(V=V, d=V, n=n, B=B, gamma=gamma, w_dtype=0, seed=1, rnd=rnd, pos=pos, W=W, H=logq[pos],
                              weights=w, temperature=np.ones(B, np.float32), draft_logits=dl, draft_lse=lse,
                              draft_tokens=tok, draft_q=dq, flags=fl)
        out = oracle.verify(V=V, n=n, B=B, gamma=gamma, distance=0, seed=1, rnd=rnd, target_logits=tl, draft_logits=dl,
                            draft_tokens=tok, draft_q=dq, weights=w, temperature=np.ones(B, np.float32))
        dev, nv = out["dev"], out["n_valid"]
        assert np.all(np.abs(w.sum(axis=1) - 1) < 1e-6)


# ------------------------------------------------------------------ two-draft grid policy (App. B.2, Alg. 1 (arg-min step))
def _grid_verify(oracle, logq, logp, distance, T=1.0):
    gamma, n, V = logq.shape
    dl = np.ascontiguousarray(logq.astype(np.float32)[:, None])      # [gamma,1,n,V]
    return oracle.verify(V=V, n=n, B=1, gamma=gamma, distance=distance, seed=0, rnd=0, n_cand=oracle.GRID_CANDIDATES,
                         target_logits=logp.astype(np.float32)[None], draft_logits=dl,
                         draft_tokens=np.zeros((1, gamma), np.int32), draft_q=np.ones((1, gamma), np.float32),
                         weights=np.full((1, n), 0.5, np.float32), temperature=np.full(1, T, np.float32))


def test_grid_candidates_are_distances_of_the_mixtures(oracle):
    rng = np.random.default_rng(31)
    V, gamma = 120, 2
    logq, logp, p, _, qj = _dists(rng, gamma, 2, V, (0.5, 0.5))
    for distance in (0, 1):
        out = _grid_verify(oracle, logq, logp, distance)
        assert out["dev"].shape == (1, gamma, 11)
        for i in range(gamma):
            ends = []
            for c in range(11):
                mix = (1 - c / 10) * qj[i, 0] + (c / 10) * qj[i, 1]
                ref = sp.rel_entr(p[i], mix).sum() if distance == 0 else 0.5 * np.abs(p[i] - mix).sum()
                assert abs(out["dev"][0, i, c] - ref) < 1e-6 * max(1.0, ref)
                ends.append(ref)
            # the end points are the per-draft distances; both distances are convex in the mixture weight
            per_draft = oracle.verify(V=V, n=2, B=1, gamma=gamma, distance=distance, seed=0, rnd=0,
                                      target_logits=logp.astype(np.float32)[None],
                                      draft_logits=np.ascontiguousarray(logq.astype(np.float32)[:, None]),
                                      draft_tokens=np.zeros((1, gamma), np.int32), draft_q=np.ones((1, gamma), np.float32),
                                      weights=np.full((1, 2), 0.5, np.float32), temperature=np.ones(1, np.float32))["dev"]
            assert abs(out["dev"][0, i, 0] - per_draft[0, i, 0]) < 1e-6 and abs(out["dev"][0, i, 10] - per_draft[0, i, 1]) < 1e-6
            for c in range(1, 10):
                assert ends[c] <= (1 - c / 10) * ends[0] + (c / 10) * ends[10] + 1e-12


def test_grid_policy_picks_the_mixture_the_target_is_made_of(oracle):
    rng = np.random.default_rng(32)
    V, gamma, h = 80, 3, 6
    for cstar in (0, 3, 7, 10):
        logq = rng.standard_normal((gamma, 2, V)) * 1.5
        qj = sp.softmax(logq.astype(np.float32).astype(np.float64), axis=-1)
        mix = (1 - cstar / 10) * qj[:, 0] + (cstar / 10) * qj[:, 1]
        logp = np.concatenate([np.log(mix), rng.standard_normal((1, V))])
        out = _grid_verify(oracle, logq, logp, 0)
        ring = np.zeros((1, h, 11), np.float32); head = np.zeros(1, np.int32); count = np.zeros(1, np.int32)
        w = oracle.update_weights(n=2, B=1, gamma=gamma, h=h, policy=2, tau_w=1.0, eps=1e-6, dev=out["dev"],
                                  n_valid=np.array([gamma], np.int32), ring=ring, ring_head=head, ring_count=count)
        np.testing.assert_allclose(w[0], [1 - cstar / 10, cstar / 10], atol=1e-7)
        assert count[0] == gamma and np.array_equal(ring[0, :gamma], out["dev"][0])


def test_grid_policy_window_ties_and_empty_window(oracle):
    ring = np.zeros((2, 4, 11), np.float32); head = np.zeros(2, np.int32); count = np.zeros(2, np.int32)
    w = oracle.update_weights(n=2, B=2, gamma=1, h=4, policy=2, tau_w=1.0, eps=1e-6, dev=None, n_valid=None,
                              ring=ring, ring_head=head, ring_count=count)
    assert np.all(w == np.float32(0.5))                        # empty window: equal weights
    dev = np.ones((2, 1, 11), np.float32)
    dev[0, 0, 4] = dev[0, 0, 8] = 0.25                         # tie between candidates 4 and 8 -> lowest index
    dev[1, 0, 10] = 0.1
    w = oracle.update_weights(n=2, B=2, gamma=1, h=4, policy=2, tau_w=1.0, eps=1e-6, dev=dev,
                              n_valid=np.array([1, 1], np.int32), ring=ring, ring_head=head, ring_count=count)
    np.testing.assert_allclose(w, [[0.6, 0.4], [0.0, 1.0]], atol=1e-7)
    # brute-force window: only the last h pushed positions count
    rng = np.random.default_rng(33)
    log = []
    ring = np.zeros((1, 3, 11), np.float32); head = np.zeros(1, np.int32); count = np.zeros(1, np.int32)
    for _ in range(12):
        dev = rng.random((1, 2, 11)).astype(np.float32)
        nv = rng.integers(1, 3, 1).astype(np.int32)
        w = oracle.update_weights(n=2, B=1, gamma=2, h=3, policy=2, tau_w=1.0, eps=1e-6, dev=dev, n_valid=nv,
                                  ring=ring, ring_head=head, ring_count=count)
        log += [dev[0, i] for i in range(nv[0])]
        c = int(np.argmin(np.sum(np.asarray(log[-3:], np.float64), axis=0)))
        np.testing.assert_allclose(w[0], [1 - c / 10, c / 10], atol=1e-7)


def test_window_all_is_the_sum_over_every_verified_position(oracle):
    """h = 0 (ALL, the paper's default window): same weights as a window longer than the run."""
    rng = np.random.default_rng(41)
    B, n, gamma = 3, 4, 5
    ring_all = np.zeros((B, 1, n), np.float32); head_a = np.zeros(B, np.int32); cnt_a = np.zeros(B, np.int32)
    ring_big = np.zeros((B, 4096, n), np.float32); head_b = np.zeros(B, np.int32); cnt_b = np.zeros(B, np.int32)
    total = np.zeros((B, n))
    for step in range(40):
        dev = (rng.random((B, gamma, n)) * 0.5 + 0.01).astype(np.float32)
        nv = rng.integers(1, gamma + 1, B).astype(np.int32)
        wa = oracle.update_weights(n=n, B=B, gamma=gamma, h=0, policy=0, tau_w=1.0, eps=1e-6, dev=dev, n_valid=nv,
                                   ring=ring_all, ring_head=head_a, ring_count=cnt_a)
        wb = oracle.update_weights(n=n, B=B, gamma=gamma, h=4096, policy=0, tau_w=1.0, eps=1e-6, dev=dev, n_valid=nv,
                                   ring=ring_big, ring_head=head_b, ring_count=cnt_b)
        for b in range(B):
            total[b] += dev[b, :nv[b]].astype(np.float64).sum(axis=0)
        np.testing.assert_allclose(wa, wb, rtol=2e-5)
        np.testing.assert_allclose(ring_all[:, 0], total, rtol=1e-5)
        assert np.array_equal(cnt_a, cnt_b)
    ring = np.zeros((1, 1, n), np.float32)
    w = oracle.update_weights(n=n, B=1, gamma=gamma, h=0, policy=0, tau_w=1.0, eps=1e-6, dev=None, n_valid=None,
                              ring=ring, ring_head=np.zeros(1, np.int32), ring_count=np.zeros(1, np.int32))
    assert np.all(w == np.float32(0.25))


def test_random_weights_are_uniform_on_the_simplex(oracle):
    """Policy 3 (the paper's random-weights ablation): Dirichlet(1,..,1), i.e. each weight ~ Beta(1, n-1),
    fresh for every block and sequence; the window is maintained all the same."""
    n, B, gamma, h = 4, 64, 3, 5
    ring = np.zeros((B, h, n), np.float32); head = np.zeros(B, np.int32); count = np.zeros(B, np.int32)
    ws = []
    for rnd in range(60):
        dev = np.full((B, gamma, n), 0.5, np.float32)
        w = oracle.update_weights(n=n, B=B, gamma=gamma, h=h, policy=3, tau_w=1.0, eps=1e-6, dev=dev if rnd else None,
                                  n_valid=np.full(B, 2, np.int32) if rnd else None, ring=ring, ring_head=head,
                                  ring_count=count, seed=9, rnd=rnd)
        assert np.all(w >= 0) and np.all(np.abs(w.sum(axis=1) - 1) < 1e-6)
        ws.append(w)
    ws = np.concatenate(ws)                                     # 3840 draws
    for j in range(n):
        assert st.kstest(ws[:, j], st.beta(1, n - 1).cdf).pvalue > 1e-3
    assert abs(ws.mean() - 1 / n) < 1e-6
    assert np.abs(np.corrcoef(ws[:-B, 0], ws[B:, 0])[0, 1]) < 0.06      # fresh per block
    assert len({tuple(r) for r in np.round(ws, 6)}) == len(ws)          # and per sequence
    assert np.all(count == h) and np.all(ring == 0.5)                   # the window was pushed all along
    # same (seed, round, b) => same weights; another seed => others
    a = oracle.update_weights(n=n, B=2, gamma=gamma, h=h, policy=3, tau_w=1.0, eps=1e-6, dev=None, n_valid=None,
                              ring=np.zeros((2, h, n), np.float32), ring_head=np.zeros(2, np.int32),
                              ring_count=np.zeros(2, np.int32), seed=9, rnd=7)
    assert np.array_equal(a, ws[7 * B: 7 * B + 2])
    b = oracle.update_weights(n=n, B=2, gamma=gamma, h=h, policy=3, tau_w=1.0, eps=1e-6, dev=None, n_valid=None,
                              ring=np.zeros((2, h, n), np.float32), ring_head=np.zeros(2, np.int32),
                              ring_count=np.zeros(2, np.int32), seed=10, rnd=7)
    assert not np.array_equal(a, b)


def test_hard_label_distance_counts_token_mismatches(oracle):
    """distance 2: 1 where the arg-max of a candidate distribution differs from the token emitted at that
    position, 0 where it matches; positions after the rejected one carry no label."""
    rng = np.random.default_rng(51)
    V, gamma = 40, 4
    for n_cand, n in ((0, 3), (11, 2)):
        for trial in range(12):
            w = rng.dirichlet(np.ones(n)).astype(np.float32)
            logq, logp, p, q, qj = _dists(rng, gamma, n, V, w)
            for i in range(trial % (gamma + 1)):                       # make the target agree on a prefix
                logp[i, int(np.argmax(q[i]))] = logp[i].max() + 2
            W = _identity_head(V)
            dl = np.ascontiguousarray(logq.astype(np.float32)[:, None])
            temp = np.zeros(1, np.float32)                             # greedy: emitted tokens are arg-maxes
            tok = np.array([[int(np.argmax(q[i])) for i in range(gamma)]], np.int32)
            out = oracle.verify(V=V, n=n, B=1, gamma=gamma, distance=2, seed=0, rnd=0, n_cand=n_cand,
                                target_logits=logp.astype(np.float32)[None], draft_logits=dl, draft_tokens=tok,
                                draft_q=np.ones((1, gamma), np.float32), weights=w[None], temperature=temp)
            k = int(out["accept_len"][0])
            cands = [qj[:, j] for j in range(n)] if n_cand == 0 else \
                    [(1 - c / 10) * qj[:, 0] + (c / 10) * qj[:, 1] for c in range(11)]
            for i in range(gamma):
                for c, dist in enumerate(cands):
                    want = 1.0 if i > k else float(int(np.argmax(dist[i])) != int(out["out_tokens"][0, i]))
                    assert out["dev"][0, i, c] == want, (n_cand, trial, i, c)
    # with the grid policy the window then prefers the candidate with the most matches
    ring = np.zeros((1, 8, 11), np.float32); head = np.zeros(1, np.int32); count = np.zeros(1, np.int32)
    dev = np.ones((1, 3, 11), np.float32); dev[0, :, 6] = 0; dev[0, 0, 2] = 0
    wts = oracle.update_weights(n=2, B=1, gamma=3, h=8, policy=2, tau_w=1.0, eps=1e-6, dev=dev,
                                n_valid=np.array([3], np.int32), ring=ring, ring_head=head, ring_count=count)
    np.testing.assert_allclose(wts[0], [0.4, 0.6], atol=1e-7)


def test_hard_label_near_tie_of_a_mixture_flags_its_position(oracle):
    """distance 2 with the two-draft grid: a candidate mixture whose two largest entries are closer than the margin
    flags every labelled position (i <= k) it occurs at and none after the rejected one; single drafts (n_cand = 0)
    are decided by their fp32 logits and never flag."""
    V, gamma = 12, 4
    SM = 2
    logq = np.full((gamma, 2, V), -3.0, np.float32)
    for i in range(gamma):
        logq[i, :, 3] = 1.0                    # both drafts put their mode on token 3 ...
    logq[1, :, 7] = 1.0                        # ... at position 1 token 7 ties with it in every mixture
    logq[3, :, 7] = 1.0                        # also at position 3, which comes after the rejection below
    logp = np.full((gamma + 1, V), -3.0, np.float32)
    logp[0, 3] = logp[1, 3] = 4.0              # the target agrees at positions 0 and 1,
    logp[2, 5] = 4.0                           # rejects at 2 (wants token 5)
    tok = np.full((1, gamma), 3, np.int32)
    args = dict(V=V, n=2, B=1, gamma=gamma, distance=2, seed=0, rnd=0, target_logits=logp[None],
                draft_logits=np.ascontiguousarray(logq[:, None]), draft_tokens=tok,
                draft_q=np.ones((1, gamma), np.float32), weights=np.full((1, 2), 0.5, np.float32),
                temperature=np.zeros(1, np.float32))
    out = oracle.verify(n_cand=oracle.GRID_CANDIDATES, **args)
    assert int(out["accept_len"][0]) == 2
    assert [int(f) & SM for f in out["flags"][0]] == [0, SM, 0, 0, 0]
    assert np.all(out["dev"][0, 1] == 0.0)     # the tie goes to the lower index, which is the label
    plain = oracle.verify(n_cand=0, **args)
    assert not np.any(plain["flags"][0] & SM)
