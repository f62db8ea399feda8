"""Pins for the oracle's token-tree functions (Sec. 6.1, "Verification: Integrating Token Tree").

The paper fixes nothing but the width, so what pins the construction is mathematics: width 1 must be the chain,
bit for bit; verification must stay lossless -- the first token a round emits follows the target distribution p_0
exactly, however many sibling candidates were tried (checked by enumerating every candidate tuple and measuring the
oracle's accept thresholds and residual draws on fine one-dimensional grids of uniforms); the token after an accepted
leaf follows the target's distribution after that leaf; greedy rows match a short independent reference."""
import itertools

import numpy as np
import pytest
import scipy.special as sp


def _setup(rng, gamma, n, V, B, width, temperature=1.0):
    S = width - 1
    logq = rng.standard_normal((gamma, n, V)).astype(np.float32) * 1.5
    logp = rng.standard_normal((gamma + 1, V)).astype(np.float32) * 1.5
    leafl = rng.standard_normal((gamma, max(S, 1), V)).astype(np.float32) * 1.5
    w = rng.dirichlet(np.ones(n)).astype(np.float32)
    return logq, logp, leafl[:, :S], w


def _mixture(logq_pos, w, T=1.0):
    """q_ens of one position from library softmax (used only to aim uniforms at chosen tokens)."""
    return (w[:, None].astype(np.float64) * sp.softmax(logq_pos.astype(np.float64) / T, axis=-1)).sum(0)


def _aim(q, token):
    """A uniform in the middle of `token`'s bin of the inverse CDF of q."""
    c = np.concatenate([[0.0], np.cumsum(q)]) / q.sum()
    return np.float32(0.5 * (c[token] + c[token + 1]))


def _round(oracle, *, logq, logp, leafl, w, width, B, temperature=1.0, seed=0, rnd=0, u_draft=None, u_sib=None,
           u_acc=None, u_res=None, u_acc_sib=None):
    """One tree round on B copies of the same distributions (identity LM head: hidden state = logit row)."""
    gamma, n, V = logq.shape
    S = width - 1
    W = np.eye(V, dtype=np.float32)
    dl = np.zeros((gamma, B, n, V), np.float32); lse = np.zeros((gamma, B, n)); tok = np.zeros((B, gamma), np.int32)
    dq = np.zeros((B, gamma), np.float32); fl = np.zeros((B, gamma), np.uint8)
    st = np.zeros((B, gamma, S), np.int32); sq = np.zeros((B, gamma, S), np.float32); sf = np.zeros((B, gamma, S), np.uint8)
    weights = np.tile(np.asarray(w, np.float32), (B, 1))
    temp = np.full(B, temperature, np.float32)
    for pos in range(gamma):
        H = np.ascontiguousarray(np.broadcast_to(logq[pos], (B, n, V)))
        oracle.draft_step(V=V, d=V, n=n, B=B, gamma=gamma, w_dtype=0, seed=seed, rnd=rnd, pos=pos, W=W, H=H,
                          weights=weights, temperature=temp, draft_logits=dl, draft_lse=lse, draft_tokens=tok,
                          draft_q=dq, flags=fl, u_draft=u_draft)
        if S:
            oracle.draft_siblings(V=V, n=n, B=B, gamma=gamma, width=width, seed=seed, rnd=rnd, pos=pos, draft_logits=dl,
                                  draft_tokens=tok, weights=weights, temperature=temp, sib_tokens=st, sib_q=sq,
                                  sib_flags=sf, u_sib=u_sib)
    tl = np.ascontiguousarray(np.broadcast_to(logp, (B, gamma + 1, V)))
    ll = np.ascontiguousarray(np.broadcast_to(leafl, (B, gamma, S, V)))
    out = oracle.verify_tree(V=V, n=n, B=B, gamma=gamma, width=width, distance=0, seed=seed, rnd=rnd, target_logits=tl,
                             leaf_logits=ll, draft_logits=dl, draft_tokens=tok, draft_q=dq, sib_tokens=st, sib_q=sq,
                             weights=weights, temperature=temp, u_acc=u_acc, u_res=u_res, u_acc_sib=u_acc_sib)
    out.update(draft_tokens=tok, draft_q=dq, sib_tokens=st, sib_q=sq, sib_flags=sf, draft_logits=dl, weights=weights, temp=temp,
               target=tl, leaf_logits=ll)
    return out


# ------------------------------------------------------------------ width 1 is the chain
def test_width_one_is_the_chain_bit_for_bit(oracle):
    rng = np.random.default_rng(5)
    for temperature in (1.0, 0.0, 0.6):
        logq, logp, leafl, w = _setup(rng, 3, 3, 9, 1, 1)
        B = 64
        t = _round(oracle, logq=logq, logp=logp, leafl=leafl, w=w, width=1, B=B, temperature=temperature, seed=3, rnd=4)
        c = oracle.verify(V=9, n=3, B=B, gamma=3, distance=0, seed=3, rnd=4, target_logits=t["target"],
                          draft_logits=t["draft_logits"], draft_tokens=t["draft_tokens"], draft_q=t["draft_q"],
                          weights=t["weights"], temperature=t["temp"])
        for key in ("accept_len", "out_tokens", "dev", "n_valid", "flags"):
            assert np.array_equal(t[key], c[key]), key
        assert np.all(t["leaf"] == 0) and np.array_equal(t["n_out"], c["accept_len"] + 1)


# ------------------------------------------------------------------ losslessness by enumeration + 1-D grids
@pytest.mark.parametrize("width", [2, 3])
def test_first_emitted_token_follows_the_target_distribution(oracle, width):
    """gamma = 1, V = 4, two drafts.  For every tuple of candidate tokens the accept probability of each candidate
    (given that the earlier ones were rejected) is measured as the measure of the accepting set of its uniform, the
    corrected token's law as the histogram over u_res; composed with the candidates' probabilities q(a) q(b) ...
    the law of the emitted token must be p_0."""
    rng = np.random.default_rng(40 + width)
    V, n, S, N = 4, 2, width - 1, 4096
    grid = ((np.arange(N) + 0.5) / N).astype(np.float32)
    for trial in range(3):
        logq, logp, leafl, w = _setup(rng, 1, n, V, 1, width)
        q = _mixture(logq[0], w)
        p0 = sp.softmax(logp[0].astype(np.float64))
        law = np.zeros(V)
        REJECT = np.float32(1.0 - 2.0 ** -24)

        def run(cands, u_acc, u_acc_sib, u_res):
            B = len(u_res)
            ud = np.full((B, 1), _aim(q, cands[0]), np.float32)
            us = np.tile(np.array([_aim(q, c) for c in cands[1:]], np.float32), (B, 1)).reshape(B, 1, S)
            out = _round(oracle, logq=logq, logp=logp, leafl=leafl, w=w, width=width, B=B, u_draft=ud, u_sib=us,
                         u_acc=np.asarray(u_acc, np.float32).reshape(B, 1),
                         u_acc_sib=np.asarray(u_acc_sib, np.float32).reshape(B, 1, S), u_res=np.asarray(u_res, np.float32))
            assert np.all(out["draft_tokens"][:, 0] == cands[0]) and np.all(out["sib_tokens"][:, 0, :] == np.array(cands[1:]))
            return out

        half = np.full(N, 0.5, np.float32)
        for cands in itertools.product(range(V), repeat=width):
            weight = float(np.prod([q[c] for c in cands]))
            # trunk
            o = run(cands, grid, np.tile(half[:, None], (1, S)), half)
            alpha = [float(np.mean(o["accept_len"] == 1))]
            # siblings, each given that everything before it was rejected
            for s in range(S):
                ua_s = np.full((N, S), REJECT, np.float32)
                ua_s[:, s] = grid
                ua_s[:, s + 1:] = 0.5
                o = run(cands, np.full(N, REJECT), ua_s, half)
                if alpha[0] == 1.0:
                    alpha.append(0.0)
                    continue
                assert np.all(o["accept_len"] == 0)
                alpha.append(float(np.mean(o["leaf"] == s + 1)))
            # corrected token once every candidate is rejected
            o = run(cands, np.full(N, REJECT), np.full((N, S), REJECT, np.float32), grid)
            resid = np.bincount(o["out_tokens"][:, 0], minlength=V) / N if alpha[0] < 1.0 else np.zeros(V)
            reach = weight
            for c, a in zip(cands, alpha):
                law[c] += reach * a
                reach *= 1.0 - a
            law += reach * resid
        np.testing.assert_allclose(law, p0, atol=4.0 / N)


def test_token_after_an_accepted_leaf_follows_its_leaf_row(oracle):
    rng = np.random.default_rng(77)
    V, n, width, N = 5, 2, 3, 16384
    S = width - 1
    logq, logp, leafl, w = _setup(rng, 2, n, V, 1, width)
    grid = ((np.arange(N) + 0.5) / N).astype(np.float32)
    # accept the trunk at position 0 (u = 0), reject it at position 1, accept sibling 2 there (its u = 0)
    u_acc = np.tile(np.array([0.0, 1.0 - 2.0 ** -24], np.float32), (N, 1))
    u_acc_sib = np.zeros((N, 2, S), np.float32)
    u_acc_sib[:, 1, 0] = 1.0 - 2.0 ** -24
    out = _round(oracle, logq=logq, logp=logp, leafl=leafl, w=w, width=width, B=N, u_acc=u_acc, u_acc_sib=u_acc_sib,
                 u_res=grid, seed=9, rnd=2)
    sel = (out["accept_len"] == 1) & (out["leaf"] == 2)
    assert sel.sum() > 300                       # u = 0 accepts wherever the residual is positive at the candidate
    assert np.all(out["n_out"][sel] == 3)
    assert np.all(out["out_tokens"][sel, 1] == out["sib_tokens"][sel, 1, 1])
    checked = 0
    for y in np.unique(out["sib_tokens"][sel, 1, 1]):         # the leaf row does not depend on the leaf token here
        pick = sel & (out["sib_tokens"][:, 1, 1] == y)
        if pick.sum() < 300:
            continue
        checked += 1
        u = grid[pick]
        hist = np.bincount(out["out_tokens"][pick, 2], minlength=V) / pick.sum()
        expect = sp.softmax(leafl[1, 1].astype(np.float64))
        # the uniforms of the selected copies are a subset of the grid: compare through the CDF they imply
        cdf = np.cumsum(expect)
        want = np.bincount(np.searchsorted(cdf, u.astype(np.float64), side="right").clip(0, V - 1), minlength=V) / pick.sum()
        np.testing.assert_allclose(hist, want, atol=3.0 / pick.sum() * V)
    assert checked >= 1


# ------------------------------------------------------------------ greedy rows against a short reference
def test_greedy_tree_matches_a_short_reference(oracle):
    rng = np.random.default_rng(13)
    for width in (2, 3):
        for trial in range(20):
            gamma, n, V = 3, 2, 7
            logq, logp, leafl, w = _setup(rng, gamma, n, V, 1, width)
            out = _round(oracle, logq=logq, logp=logp, leafl=leafl, w=w, width=width, B=1, temperature=0.0)
            emitted, leaf = [], 0
            for i in range(gamma + 1):
                if i == gamma:
                    emitted.append(int(np.argmax(logp[gamma])))
                    break
                order = np.argsort(-_mixture(logq[i], w), kind="stable")[:width]      # top `width`, lowest index on ties
                top = int(np.argmax(logp[i]))
                assert out["draft_tokens"][0, i] == order[0] and list(out["sib_tokens"][0, i]) == list(order[1:])
                if order[0] == top:
                    emitted.append(top)
                    continue
                emitted.append(top)
                hit = [s for s in range(1, width) if order[s] == top]
                if hit:
                    leaf = hit[0]
                    emitted.append(int(np.argmax(leafl[i, leaf - 1])))
                break
            k = out["accept_len"][0]
            assert out["leaf"][0] == leaf and out["n_out"][0] == len(emitted)
            assert list(out["out_tokens"][0, :len(emitted)]) == emitted
            assert np.all(out["out_tokens"][0, len(emitted):] == -1)
            assert out["n_valid"][0] == min(k + 1, gamma)


# ------------------------------------------------------------------ structure: uniforms, distances, counts
def test_sibling_uniforms_are_their_own_philox_blocks_and_distances_are_the_chains(oracle):
    rng = np.random.default_rng(21)
    gamma, n, V, width, B = 3, 3, 11, 3, 128
    S = width - 1
    logq, logp, leafl, w = _setup(rng, gamma, n, V, 1, width)
    seed, rnd = 0xABCDEF12345, 17
    a = _round(oracle, logq=logq, logp=logp, leafl=leafl, w=w, width=width, B=B, seed=seed, rnd=rnd)
    u = lambda pos, word: np.array([oracle.uniform(seed, rnd, b, pos, word) for b in range(B)], np.float32)
    ud = np.stack([u(i, 0) for i in range(gamma)], 1)
    ua = np.stack([u(i, 1) for i in range(gamma)], 1)
    us = np.stack([np.stack([u(i + s * oracle.SIB_STRIDE, 0) for s in range(1, width)], 1) for i in range(gamma)], 1)
    uas = np.stack([np.stack([u(i + s * oracle.SIB_STRIDE, 1) for s in range(1, width)], 1) for i in range(gamma)], 1)
    b = _round(oracle, logq=logq, logp=logp, leafl=leafl, w=w, width=width, B=B, seed=seed + 1, rnd=rnd + 1,
               u_draft=ud, u_sib=us, u_acc=ua, u_acc_sib=uas, u_res=u(gamma, 0))
    for key in ("accept_len", "out_tokens", "leaf", "n_out", "sib_tokens", "draft_tokens", "flags"):
        assert np.array_equal(a[key], b[key]), key
    assert len(set(np.concatenate([ud.ravel(), ua.ravel(), us.ravel(), uas.ravel()]).tolist())) > 0.99 * (ud.size * 2 + us.size * 2)
    c = oracle.verify(V=V, n=n, B=B, gamma=gamma, distance=0, seed=seed, rnd=rnd, target_logits=a["target"],
                      draft_logits=a["draft_logits"], draft_tokens=a["draft_tokens"], draft_q=a["draft_q"],
                      weights=a["weights"], temperature=a["temp"])
    assert np.array_equal(a["dev"], c["dev"]) and np.array_equal(a["n_valid"], c["n_valid"])
    assert np.array_equal(a["accept_len"], c["accept_len"])
    assert np.all(a["n_out"] == a["accept_len"] + 1 + (a["leaf"] > 0))
    assert (a["leaf"] > 0).any() and (a["leaf"] == 0).any()
    # a tree never emits fewer tokens than the chain on the same inputs
    assert a["n_out"].mean() >= (c["accept_len"] + 1).mean()
