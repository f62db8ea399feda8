"""Shared machinery of the GPU parity tests: run SD rounds through the C ABI (via the binding) and through
the CPU oracle on the same seeded inputs, and compare element by element.

Tolerances, and where they come from (the oracle computes in fp64 from the same stored inputs):
  logits        |dL| <= 1e-5 * max|L| and <= 2e-2: bf16 x bf16 products are exact in fp32, the MFMA adds d of them in
                fp32, so the error is ~d * eps * |terms| ~ 1e-6 at |L| ~ 1
  lse           |d| <= 2e-6 absolute (a logit error moves a log-sum-exp by at most that error)
  q(y), p       relative 1e-5 (a logit error delta moves a log-probability by at most 2 * delta)
  dev           |d| <= 1e-5 * |dev| + 1e-6: KL is a difference of O(1)..O(10) quantities, so its error is absolute
  weights       |d| <= 1e-5 * w + 1e-6 end to end (x = 1/e amplifies an absolute error of e by 1/e^2); the weights
                kernel alone, fed identical windows, is tested to 1e-6 relative
  integers      bit-exact unless the decision that produced them is flagged (margin < 1e-6) on either side
"""
from __future__ import annotations

import numpy as np
import torch

from paper_2601_20357_amd import binding, synth

DEV = "cuda:0"


def to_dev_store(x: np.ndarray, w_dtype: int) -> torch.Tensor:
    """Storage array (fp32 or bf16 bit patterns) -> device tensor of the matching torch dtype."""
    if w_dtype == 0:
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).to(DEV).view(torch.bfloat16)


def cfg_of(wl: synth.Workload, seed=0, policy=0, tau_w=1.0, eps=1e-6, distance=0):
    return binding.make_cfg(V=wl.V, d=wl.d, n=wl.n, B=wl.B, gamma=wl.gamma, h=wl.h, w_dtype=wl.w_dtype,
                            policy=policy, tau_w=tau_w, eps=eps, seed=seed, distance=distance)


class OracleSide:
    def __init__(self, oracle, wl, seed=0, policy=0, tau_w=1.0, eps=1e-6, distance=0):
        self.o, self.wl, self.seed, self.policy, self.tau_w, self.eps = oracle, wl, seed, policy, tau_w, eps
        self.distance = distance
        B, n, g, h, V = wl.B, wl.n, wl.gamma, wl.h, wl.V
        self.ring = np.zeros((B, max(h, 1), oracle.dev_width(n, policy)), np.float32)
        self.head = np.zeros(B, np.int32)
        self.count = np.zeros(B, np.int32)
        self.dev = None
        self.n_valid = None

    def round(self, rnd, W, H, target, temp, u_draft=None, u_acc=None, u_res=None):
        wl, o = self.wl, self.o
        B, n, g, V = wl.B, wl.n, wl.gamma, wl.V
        w = o.update_weights(n=n, B=B, gamma=g, h=wl.h, policy=self.policy, tau_w=self.tau_w, eps=self.eps,
                             dev=self.dev, n_valid=self.n_valid, ring=self.ring, ring_head=self.head,
                             ring_count=self.count, seed=self.seed, rnd=rnd)
        dl = np.zeros((g, B, n, V), np.float32)
        lse = np.zeros((g, B, n), np.float64)
        tok = np.zeros((B, g), np.int32)
        dq = np.zeros((B, g), np.float32)
        fl = np.zeros((B, g), np.uint8)
        for pos in range(g):
            o.draft_step(V=V, d=wl.d, n=n, B=B, gamma=g, w_dtype=wl.w_dtype, seed=self.seed, rnd=rnd, pos=pos, W=W,
                         H=H[pos], weights=w, temperature=temp, draft_logits=dl, draft_lse=lse, draft_tokens=tok,
                         draft_q=dq, flags=fl, u_draft=u_draft)
        out = o.verify(V=V, n=n, B=B, gamma=g, distance=self.distance, seed=self.seed, rnd=rnd, target_logits=target,
                       draft_logits=dl, draft_tokens=tok, draft_q=dq, weights=w, temperature=temp, u_acc=u_acc,
                       u_res=u_res, n_cand=o.GRID_CANDIDATES if self.policy == 2 else 0)
        self.dev, self.n_valid = out["dev"], out["n_valid"]
        out.update(weights=w, draft_logits=dl, draft_lse=lse, draft_tokens=tok, draft_q=dq, draft_flags=fl)
        return out


class GpuSide:
    def __init__(self, wl, seed=0, policy=0, tau_w=1.0, eps=1e-6, distance=0, fused=False):
        self.wl = wl
        self.cfg = cfg_of(wl, seed, policy, tau_w, eps, distance)
        self.buf = binding.RoundBuffers(self.cfg, DEV)
        self.first = True
        self.fused = fused          # tabed_verify also opens the next round (window push + next weights)
        self.need_update = True

    def round(self, rnd, W_t, H, target, temp, u_draft=None, u_acc=None, u_res=None, rows=None):
        """rows: indices of the sequences whose results are copied back (default: all of them)."""
        wl, buf = self.wl, self.buf
        t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)
        temp_t, tgt_t = t(temp), t(target)
        ud, ua, ur = t(u_draft), t(u_acc), t(u_res)
        if self.need_update:
            buf.update_weights(self.first, rnd=rnd)
        self.first = False
        self.need_update = not self.fused
        w_used = buf.weights.clone()
        for pos in range(wl.gamma):
            buf.draft_step(rnd, pos, W_t, to_dev_store(H[pos], wl.w_dtype), temp_t, ud)
        buf.verify(rnd, tgt_t, temp_t, ua, ur, fused_update=self.fused)
        torch.cuda.synchronize()
        if rows is None:
            c = lambda x: x.cpu().numpy()
            c1 = c
        else:
            idx = torch.as_tensor(np.asarray(rows), device=DEV, dtype=torch.long)
            c = lambda x: x.index_select(0, idx).cpu().numpy()       # [B, ...]
            c1 = lambda x: x.index_select(1, idx).cpu().numpy()      # [gamma, B, ...]
        return dict(weights=c(w_used), draft_logits=c1(buf.draft_logits), draft_lse=c1(buf.draft_lse),
                    draft_tokens=c(buf.draft_tokens), draft_q=c(buf.draft_q), draft_flags=c(buf.draft_flags),
                    accept_len=c(buf.accept_len), out_tokens=c(buf.out_tokens), dev=c(buf.dev),
                    n_valid=c(buf.n_valid), flags=c(buf.verify_flags))

    def resync_from(self, orc: OracleSide, rows=None):
        """After a flagged divergence: continue from the oracle's window state (HIP input <- oracle is allowed).
        rows: the sequences the oracle ran (default: all of them)."""
        idx = slice(None) if rows is None else torch.as_tensor(np.asarray(rows), device=DEV, dtype=torch.long)
        self.buf.ring[idx] = torch.from_numpy(orc.ring).to(DEV)
        self.buf.ring_head[idx] = torch.from_numpy(orc.head).to(DEV)
        self.buf.ring_count[idx] = torch.from_numpy(orc.count).to(DEV)
        self.buf.dev[idx] = torch.from_numpy(orc.dev).to(DEV)
        self.buf.n_valid[idx] = torch.from_numpy(orc.n_valid).to(DEV)
        if rows is not None and not self.need_update:
            raise AssertionError("a subset resync needs the separate window update (fused=False)")
        self.need_update = True     # fused mode: redo the push from the oracle's distances with the plain call


class Tally:
    def __init__(self):
        self.decisions = 0
        self.flagged_divergences = 0
        self.max_logit_err = 0.0
        self.max_q_rel = 0.0
        self.max_dev_err = 0.0
        self.max_w_err = 0.0
        self.gpu_flags = 0          # decisions the GPU flagged as closer than 1e-6
        self.oracle_flags = 0
        self.gpu_only_flags = 0     # ... that the oracle did not flag (its own margin is then checked)
        self.max_gpu_only_margin = 0.0

    def count_flag(self, g_flag, o_flag, margin_fn):
        """Book-keeping of one decision's margin flags.  A flag the GPU raises alone must correspond to a real
        near-tie: the oracle-side margin of the same decision (fp64) has to be below 1e-5."""
        self.gpu_flags += bool(g_flag)
        self.oracle_flags += bool(o_flag)
        if g_flag and not o_flag and margin_fn is not None:
            m = float(margin_fn())
            self.gpu_only_flags += 1
            self.max_gpu_only_margin = max(self.max_gpu_only_margin, m)
            assert m < 1e-5, f"the GPU flagged a decision whose oracle-side margin is {m:.3e}"

    def __repr__(self):
        return (f"decisions={self.decisions} flagged_divergences={self.flagged_divergences} "
                f"gpu_flags={self.gpu_flags} oracle_flags={self.oracle_flags} gpu_only_flags={self.gpu_only_flags} "
                f"max|dL|={self.max_logit_err:.2e} max rel dq={self.max_q_rel:.2e} "
                f"max|ddev|={self.max_dev_err:.2e} max|dw|={self.max_w_err:.2e}")


class Margins:
    """Oracle-side margin (fp64) of a decision of one round, computed on request from the oracle's own building
    blocks: how close the decision was to going the other way, in the units the flags use."""

    def __init__(self, oracle, wl, o, target, temp, seed, rnd, b_index, u_draft=None, u_acc=None, u_res=None):
        self.o_, self.wl, self.o, self.target, self.temp = oracle, wl, o, target, temp
        self.seed, self.rnd, self.b_index = seed, rnd, b_index      # b_index[b] = the sequence's Philox stream
        self.u_draft, self.u_acc, self.u_res = u_draft, u_acc, u_res

    def _t_eff(self, b):
        return float(self.temp[b]) if self.temp[b] > 0 else 1.0

    def _q_ens(self, b, pos):
        o, wl = self.o_, self.wl
        q = np.stack([o.softmax(self.o["draft_logits"][pos, b, j], self._t_eff(b))[0] for j in range(wl.n)])
        return o.ensemble(q, self.o["weights"][b])

    @staticmethod
    def _cdf_margin(f, u, tok):
        Z = float(f.sum())
        cdf = np.cumsum(f)
        m = np.inf
        if tok + 1 < len(f):
            m = min(m, abs(cdf[tok] - u * Z))
        if tok > 0:
            m = min(m, abs(cdf[tok - 1] - u * Z))
        return m / Z

    def draft(self, b, pos):
        f = self._q_ens(b, pos)
        if not self.temp[b] > 0:
            top = np.sort(f)[-2:]
            return (top[1] - top[0]) / abs(top[1])
        u = self.u_draft[b, pos] if self.u_draft is not None else self.o_.uniform(self.seed, self.rnd, int(self.b_index[b]), pos, 0)
        return self._cdf_margin(f, float(u), int(self.o["draft_tokens"][b, pos]))

    def accept(self, b, i):
        y = int(self.o["draft_tokens"][b, i])
        p = self.o_.softmax(self.target[b, i], self._t_eff(b))[0]
        u = self.u_acc[b, i] if self.u_acc is not None else self.o_.uniform(self.seed, self.rnd, int(self.b_index[b]), i, 1)
        lhs, py = float(np.float32(u) * np.float32(self.o["draft_q"][b, i])), float(np.float32(p[y]))
        return abs(lhs - py) / max(lhs, py)

    def emitted(self, b, k):
        p = self.o_.softmax(self.target[b, k], self._t_eff(b))[0]
        f = p if k == self.wl.gamma else np.maximum(0.0, p - self._q_ens(b, k))
        if not f.sum() > 0:
            return 0.0
        u = self.u_res[b] if self.u_res is not None else self.o_.uniform(self.seed, self.rnd, int(self.b_index[b]), self.wl.gamma, 0)
        return self._cdf_margin(f, float(u), int(self.o["out_tokens"][b, k]))


def compare_round(g, o, wl, tally: Tally, check_logits=True, hard=False, margins: Margins | None = None, grid_tie=None):
    """Element-by-element comparison of one round (wl: the workload of the sequences compared).  Returns True
    if every sequence stayed in lock-step; False if a flagged decision diverged (the caller then resyncs the
    window state).

    grid_tie(b, c_gpu, c_oracle): two-draft grid policy only.  Its weights are an arg-min over 11 window sums of fp32
    distances that differ between the two sides in their last bits; when two candidates' sums are closer than the
    tolerance of the distances themselves the arg-min may legitimately differ.  The callback says whether the
    oracle-side sums of the two candidates are that close; the sequence is then not compared in this round."""
    B, n, gamma = wl.B, wl.n, wl.gamma
    SM, AM = binding.FLAG_SAMPLE_MARGIN, binding.FLAG_ACCEPT_MARGIN
    skip = set()
    if grid_tie is not None:
        for b in range(B):
            if not np.array_equal(g["weights"][b], o["weights"][b]):
                c_g, c_o = int(round(float(g["weights"][b, 1]) * 10)), int(round(float(o["weights"][b, 1]) * 10))
                assert abs(float(g["weights"][b, 1]) - c_g / 10) < 1e-6 and grid_tie(b, c_g, c_o), \
                    f"grid weights differ without a tie b={b}: {g['weights'][b]} vs {o['weights'][b]}"
                skip.add(b)
                tally.flagged_divergences += 1
    same = [b for b in range(B) if b not in skip]
    np.testing.assert_allclose(g["weights"][same], o["weights"][same], rtol=1e-5, atol=1e-6)
    if same:
        tally.max_w_err = max(tally.max_w_err, float(np.max(np.abs(g["weights"][same] - o["weights"][same]))))
    if check_logits:
        scale = float(np.max(np.abs(o["draft_logits"])))
        err = float(np.max(np.abs(g["draft_logits"] - o["draft_logits"])))
        tally.max_logit_err = max(tally.max_logit_err, err)
        assert err <= 1e-5 * max(scale, 1.0) and err <= 2e-2, (err, scale)
    np.testing.assert_allclose(g["draft_lse"], o["draft_lse"], rtol=0, atol=2e-6)
    lock = not skip
    for b in same:
        alive = True      # this sequence still comparable in this round
        for pos in range(gamma):
            tally.decisions += 1
            tally.count_flag(g["draft_flags"][b, pos] & SM, o["draft_flags"][b, pos] & SM,
                             (lambda b=b, pos=pos: margins.draft(b, pos)) if margins else None)
            if g["draft_tokens"][b, pos] != o["draft_tokens"][b, pos]:
                flagged = (g["draft_flags"][b, pos] | o["draft_flags"][b, pos]) & SM
                assert flagged, f"unflagged draft token mismatch b={b} pos={pos}: {g['draft_tokens'][b]} vs {o['draft_tokens'][b]}"
                tally.flagged_divergences += 1
                alive = False
                break
            rel = abs(float(g["draft_q"][b, pos]) - float(o["draft_q"][b, pos])) / max(float(o["draft_q"][b, pos]), 1e-30)
            tally.max_q_rel = max(tally.max_q_rel, rel)
            assert rel <= 1e-5, (b, pos, g["draft_q"][b, pos], o["draft_q"][b, pos])
        # KL / TVD distances do not depend on any decision: always comparable.  Hard-label distances depend on
        # the emitted tokens: they are compared below, once the sequence is known to be in lock-step.
        d_g, d_o = g["dev"][b], o["dev"][b]
        if not hard:
            derr = np.abs(d_g - d_o)
            tally.max_dev_err = max(tally.max_dev_err, float(derr.max()))
            assert np.all(derr <= 1e-5 * np.abs(d_o) + 1e-6), (b, d_g, d_o)
        if not alive:
            lock = False
            continue
        tally.decisions += 1
        kg, ko = int(g["accept_len"][b]), int(o["accept_len"][b])
        for i in range(min(min(kg, ko) + 1, gamma)):       # accept tests both sides evaluated
            tally.count_flag(g["flags"][b, i] & AM, o["flags"][b, i] & AM,
                             (lambda b=b, i=i: margins.accept(b, i)) if margins else None)
        if kg != ko:
            i = min(kg, ko)
            flagged = (g["flags"][b, i] | o["flags"][b, i]) & AM
            assert flagged, f"unflagged accept-length mismatch b={b}: {kg} vs {ko}"
            tally.flagged_divergences += 1
            lock = False
            continue
        assert g["n_valid"][b] == o["n_valid"][b] == min(ko + 1, gamma)
        assert np.array_equal(g["out_tokens"][b, :ko], o["out_tokens"][b, :ko])
        assert np.all(g["out_tokens"][b, ko + 1:] == -1)
        tally.decisions += 1
        # (with hard labels the bit at ko can also stand for a near-tie among the mixtures' arg-maxes: no margin check)
        tally.count_flag(g["flags"][b, ko] & SM, o["flags"][b, ko] & SM,
                         (lambda b=b, ko=ko: margins.emitted(b, ko)) if margins and not hard else None)
        if g["out_tokens"][b, ko] != o["out_tokens"][b, ko]:
            flagged = (g["flags"][b, ko] | o["flags"][b, ko]) & SM
            assert flagged, f"unflagged emitted-token mismatch b={b} k={ko}: {g['out_tokens'][b]} vs {o['out_tokens'][b]}"
            tally.flagged_divergences += 1
            # the emitted token does not enter the window state (unless it is a hard label): still in lock-step
            if hard:
                lock = False
        elif hard:
            # mismatch indicators: exact, except at a labelled position one side flagged for a near-tie between the
            # two largest entries of a candidate mixture (evaluated in fp32 on one side, fp64 on the other)
            differ = np.any(d_g != d_o, axis=1)
            tied = ((g["flags"][b, :gamma] | o["flags"][b, :gamma]) & SM) != 0
            assert not np.any(differ & ~tied), (b, d_g, d_o, g["flags"][b], o["flags"][b])
            if np.any(differ):
                tally.flagged_divergences += 1
                lock = False
    return lock


def run_rounds(oracle, wl, rounds, temp, seed=0, policy=0, check_logits=True, uniforms=None, W=None, distance=0,
               fused=False, start_round=0, rows=None, on_round=None, max_gpu_flags=None):
    """Drive both sides for `rounds` rounds with state carried over; returns the tally.

    rows: the GPU runs all wl.B sequences, the oracle only these (sequences are independent: each has its own
    window, weights, temperature and Philox stream b); their results are compared element by element.
    on_round(rnd, g, o): extra assertions of the caller on the two sides' outputs (those sequences only).
    Besides the comparison itself the run asserts that the GPU raises margin flags only on real near-ties: every
    flag the oracle does not raise too is checked against the oracle-side margin of that decision (count_flag),
    and there are few of those (at most max_gpu_flags, default 1 % of the decisions, never fewer than 2 allowed).
    (Flags as such are not rare on flat distributions: with probabilities around 1/V = 2.5e-5 a uniform lands
    within 1e-6 of a bin edge in 8 % of the draws, on both sides alike.)"""
    W = synth.make_lm_head(wl) if W is None else W
    W_t = to_dev_store(W, wl.w_dtype)
    b_index = np.arange(wl.B) if rows is None else np.asarray(rows)
    wl_o = wl if rows is None else synth.scaled(wl, B=len(b_index))
    assert rows is None or (policy != 3 and not fused), "a subset run needs per-sequence state only"
    orc = OracleSide(oracle, wl_o, seed, policy, distance=distance)
    gpu = GpuSide(wl, seed, policy, distance=distance, fused=fused)
    tally = Tally()
    for rnd in range(start_round, start_round + rounds):
        H, target = synth.make_round(wl, W, rnd)
        u = uniforms(rnd) if uniforms else {}
        g = gpu.round(rnd, W_t, H, target, temp, rows=rows, **u)
        if rows is None:
            H_o, target_o, temp_o, u_o = H, target, temp, u
        else:
            # the oracle sees the subset as sequences 0..len-1, so its Philox streams are handed over explicitly:
            # the uniforms of the ORIGINAL sequence indices, drawn from the oracle's own generator
            assert not u, "explicit uniforms and a subset are not combined"
            H_o, target_o, temp_o = np.ascontiguousarray(H[:, b_index]), np.ascontiguousarray(target[b_index]), temp[b_index]
            g_ = wl.gamma
            u_o = dict(u_draft=np.array([[oracle.uniform(seed, rnd, int(b), p, 0) for p in range(g_)] for b in b_index], np.float32),
                       u_acc=np.array([[oracle.uniform(seed, rnd, int(b), p, 1) for p in range(g_)] for b in b_index], np.float32),
                       u_res=np.array([oracle.uniform(seed, rnd, int(b), g_, 0) for b in b_index], np.float32))
        o = orc.round(rnd, W, H_o, target_o, temp_o, **u_o)
        margins = Margins(oracle, wl_o, o, target_o, temp_o, seed, rnd, b_index, **{k: u_o.get(k) for k in ("u_draft", "u_acc", "u_res")})
        grid_tie = None
        if policy == 2:
            def grid_tie(b, c_g, c_o, orc=orc):
                live = orc.ring[b, :max(int(orc.count[b]), 1)].astype(np.float64) if wl.h > 0 else orc.ring[b, :1].astype(np.float64)
                e = live.sum(axis=0)
                return abs(e[c_g] - e[c_o]) <= 1e-5 * abs(e[c_o]) + 1e-6 * live.shape[0]
        if not compare_round(g, o, wl_o, tally, check_logits, hard=(distance == 2), margins=margins, grid_tie=grid_tie):
            gpu.resync_from(orc, rows)
        if on_round is not None:
            on_round(rnd, g, o)
    limit = max(2, tally.decisions // 100) if max_gpu_flags is None else max_gpu_flags
    assert tally.gpu_only_flags <= limit, f"the GPU alone flagged {tally.gpu_only_flags} of {tally.decisions} decisions"
    return tally


# ---------------------------------------------------------------- token tree (Sec. 6.1)
def run_rounds_tree(oracle, wl, rounds, temp, width, seed=0, distance=0, fused=False, explicit_uniforms=False, policy=0):
    """Both sides draft a width-`width` token tree (trunk + siblings per position) and verify it, state carried
    over `rounds` rounds.  The trunk is compared by compare_round; on top of it the siblings (token, q, flags),
    the accepted leaf, the number of emitted tokens and the tokens at and after the stopping position."""
    S = width - 1
    B, n, g, V, h = wl.B, wl.n, wl.gamma, wl.V, wl.h
    W = synth.make_lm_head(wl)
    W_t = to_dev_store(W, wl.w_dtype)
    orc = OracleSide(oracle, wl, seed, policy, distance=distance)
    cfg = cfg_of(wl, seed, policy=policy, distance=distance)
    buf = binding.RoundBuffers(cfg, DEV)
    zi = lambda shape, dt: torch.zeros(shape, dtype=dt, device=DEV)
    sib_tok, sib_q, sib_fl = zi((B, g, max(S, 1)), torch.int32), zi((B, g, max(S, 1)), torch.float32), zi((B, g, max(S, 1)), torch.uint8)
    leaf_t, nout_t = zi((B,), torch.int32), zi((B,), torch.int32)
    next_w = zi((B, n), torch.float32)
    tally = Tally()
    SM, AM = binding.FLAG_SAMPLE_MARGIN, binding.FLAG_ACCEPT_MARGIN
    first, need_update = True, True
    rng = np.random.default_rng(777 + seed)
    for rnd in range(rounds):
        H, target = synth.make_round(wl, W, rnd)
        leaves = synth.make_tree_leaves(wl, W, H, rnd, width) if S else np.zeros((B, g, 0, V), np.float32)
        u = {}
        if explicit_uniforms:
            u = dict(u_draft=rng.random((B, g), dtype=np.float32), u_acc=rng.random((B, g), dtype=np.float32),
                     u_res=rng.random(B, dtype=np.float32), u_sib=rng.random((B, g, S), dtype=np.float32),
                     u_acc_sib=rng.random((B, g, S), dtype=np.float32))
        # ---- oracle
        w_o = oracle.update_weights(n=n, B=B, gamma=g, h=h, policy=policy, tau_w=1.0, eps=1e-6, dev=orc.dev, n_valid=orc.n_valid,
                                    ring=orc.ring, ring_head=orc.head, ring_count=orc.count, seed=seed, rnd=rnd)
        dl = np.zeros((g, B, n, V), np.float32); lse = np.zeros((g, B, n)); tok = np.zeros((B, g), np.int32)
        dq = np.zeros((B, g), np.float32); fl = np.zeros((B, g), np.uint8)
        o_st = np.zeros((B, g, S), np.int32); o_sq = np.zeros((B, g, S), np.float32); o_sf = np.zeros((B, g, S), np.uint8)
        for pos in range(g):
            oracle.draft_step(V=V, d=wl.d, n=n, B=B, gamma=g, w_dtype=wl.w_dtype, seed=seed, rnd=rnd, pos=pos, W=W, H=H[pos],
                              weights=w_o, temperature=temp, draft_logits=dl, draft_lse=lse, draft_tokens=tok, draft_q=dq,
                              flags=fl, u_draft=u.get("u_draft"))
            if S:
                oracle.draft_siblings(V=V, n=n, B=B, gamma=g, width=width, seed=seed, rnd=rnd, pos=pos, draft_logits=dl,
                                      draft_tokens=tok, weights=w_o, temperature=temp, sib_tokens=o_st, sib_q=o_sq,
                                      sib_flags=o_sf, u_sib=u.get("u_sib"))
        o = oracle.verify_tree(V=V, n=n, B=B, gamma=g, width=width, distance=distance, seed=seed, rnd=rnd, target_logits=target,
                               leaf_logits=leaves, draft_logits=dl, draft_tokens=tok, draft_q=dq, sib_tokens=o_st, sib_q=o_sq,
                               weights=w_o, temperature=temp, u_acc=u.get("u_acc"), u_res=u.get("u_res"),
                               u_acc_sib=u.get("u_acc_sib"))
        orc.dev, orc.n_valid = o["dev"], o["n_valid"]
        o.update(weights=w_o, draft_logits=dl, draft_lse=lse, draft_tokens=tok, draft_q=dq, draft_flags=fl)
        # ---- GPU
        t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)
        temp_t, tgt_t, leaves_t = t(temp), t(target), t(leaves)
        ug = {k: t(v) for k, v in u.items()}
        if need_update:
            buf.update_weights(first, rnd=rnd)
        first, need_update = False, not fused
        w_used = buf.weights.clone()
        for pos in range(g):
            buf.draft_step(rnd, pos, W_t, to_dev_store(H[pos], wl.w_dtype), temp_t, ug.get("u_draft"))
            if S:
                binding.tabed_draft_siblings(cfg, buf.ws, rnd, pos, width, buf.draft_logits, buf.draft_tokens, buf.weights,
                                             temp_t, sib_tok, sib_q, sib_fl, u_sib=ug.get("u_sib"))
        win = dict(ring=buf.ring, ring_head=buf.ring_head, ring_count=buf.ring_count, next_weights=next_w) if fused else {}
        binding.tabed_verify_tree(cfg, buf.ws, rnd, width, tgt_t, leaves_t if S else None, buf.draft_logits, buf.draft_lse,
                                  buf.draft_tokens, buf.draft_q, sib_tok if S else None, sib_q if S else None, buf.weights,
                                  temp_t, buf.accept_len, buf.out_tokens, buf.dev, buf.n_valid, buf.verify_flags, leaf_t,
                                  nout_t, u_acc=ug.get("u_acc"), u_res=ug.get("u_res"), u_acc_sib=ug.get("u_acc_sib"), **win)
        torch.cuda.synchronize()
        if fused:
            buf.weights.copy_(next_w)
        c = lambda x: x.cpu().numpy()
        gd = dict(weights=c(w_used), draft_logits=c(buf.draft_logits), draft_lse=c(buf.draft_lse), draft_tokens=c(buf.draft_tokens),
                  draft_q=c(buf.draft_q), draft_flags=c(buf.draft_flags), accept_len=c(buf.accept_len), out_tokens=c(buf.out_tokens),
                  dev=c(buf.dev), n_valid=c(buf.n_valid), flags=c(buf.verify_flags))
        g_st, g_sq, g_sf, g_leaf, g_nout = c(sib_tok)[:, :, :S], c(sib_q)[:, :, :S], c(sib_fl)[:, :, :S], c(leaf_t), c(nout_t)
        # ---- the walk beyond the trunk, sequence by sequence
        lock = True
        np.testing.assert_allclose(gd["weights"], o["weights"], rtol=1e-5, atol=1e-6)
        err = float(np.max(np.abs(gd["draft_logits"] - o["draft_logits"])))
        assert err <= 1e-5 * max(float(np.max(np.abs(o["draft_logits"]))), 1.0)
        tally.max_logit_err = max(tally.max_logit_err, err)
        np.testing.assert_allclose(gd["draft_lse"], o["draft_lse"], rtol=0, atol=2e-6)
        derr = np.abs(gd["dev"] - o["dev"])
        assert np.all(derr <= 1e-5 * np.abs(o["dev"]) + 1e-6)
        tally.max_dev_err = max(tally.max_dev_err, float(derr.max()))
        for b in range(B):
            ok = True
            for pos in range(g):                      # candidates: trunk, then siblings
                cands = [(gd["draft_tokens"][b, pos], o["draft_tokens"][b, pos], gd["draft_q"][b, pos], o["draft_q"][b, pos],
                          gd["draft_flags"][b, pos] | o["draft_flags"][b, pos])]
                cands += [(g_st[b, pos, s], o_st[b, pos, s], g_sq[b, pos, s], o_sq[b, pos, s], g_sf[b, pos, s] | o_sf[b, pos, s])
                          for s in range(S)]
                for tg, to, qg, qo, fboth in cands:
                    tally.decisions += 1
                    if tg != to:
                        assert fboth & SM, f"unflagged candidate mismatch b={b} pos={pos}: {tg} vs {to}"
                        tally.flagged_divergences += 1
                        ok = False
                        break
                    assert abs(float(qg) - float(qo)) <= 1e-5 * float(qo), (b, pos, qg, qo)
                if not ok:
                    break
            if not ok:
                lock = False
                continue
            tally.decisions += 1
            kg, ko = int(gd["accept_len"][b]), int(o["accept_len"][b])
            if kg != ko:
                assert (gd["flags"][b, min(kg, ko)] | o["flags"][b, min(kg, ko)]) & AM, f"unflagged accept-length mismatch b={b}: {kg} vs {ko}"
                tally.flagged_divergences += 1
                lock = False
                continue
            assert gd["n_valid"][b] == o["n_valid"][b] == min(ko + 1, g)
            assert np.array_equal(gd["out_tokens"][b, :ko], o["out_tokens"][b, :ko])
            fk = int(gd["flags"][b, min(ko, g)] | o["flags"][b, min(ko, g)])
            if g_leaf[b] != o["leaf"][b]:
                assert fk & AM, f"unflagged sibling decision mismatch b={b} k={ko}: leaf {g_leaf[b]} vs {o['leaf'][b]}"
                tally.flagged_divergences += 1
                continue
            assert g_nout[b] == o["n_out"][b] == ko + 1 + (1 if o["leaf"][b] else 0)
            m = int(o["n_out"][b])
            assert np.all(gd["out_tokens"][b, m:] == -1) and np.all(o["out_tokens"][b, m:] == -1)
            for col in range(ko, m):
                tally.decisions += 1
                if gd["out_tokens"][b, col] != o["out_tokens"][b, col]:
                    fcol = int(gd["flags"][b, col] | o["flags"][b, col])
                    assert fcol & SM, f"unflagged emitted-token mismatch b={b} col={col}: {gd['out_tokens'][b]} vs {o['out_tokens'][b]}"
                    tally.flagged_divergences += 1
        tally.leaves = getattr(tally, "leaves", 0) + int((o["leaf"] > 0).sum())
        tally.emitted = getattr(tally, "emitted", 0) + int(o["n_out"].sum())
        if not lock:
            buf.ring.copy_(torch.from_numpy(orc.ring).to(DEV)); buf.ring_head.copy_(torch.from_numpy(orc.head).to(DEV))
            buf.ring_count.copy_(torch.from_numpy(orc.count).to(DEV)); buf.dev.copy_(torch.from_numpy(orc.dev).to(DEV))
            buf.n_valid.copy_(torch.from_numpy(orc.n_valid).to(DEV))
            need_update = True
    return tally
