"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2601_20357_amd import binding, synth

import harness
from harness import DEV

pytestmark = pytest.mark.gpu

TINY = synth.WORKLOADS["tiny"]
SERVING = synth.WORKLOADS["serving"]


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ Philox: two implementations, same bits
def test_philox_uniforms_bit_equal_to_oracle(oracle):
    cfg = binding.make_cfg(V=8, d=8, n=1, B=64, gamma=15, h=1, w_dtype=0, seed=0x123456789ABCDEF)
    out = torch.zeros((64, 16, 2), dtype=torch.float32, device=DEV)
    for rnd in (0, 1, 77, (1 << 40) + 5):
        binding.tabed_philox_uniforms(cfg, rnd, out)
        got = out.cpu().numpy()
        ref = np.array([[[oracle.uniform(cfg.seed, rnd, b, p, w) for w in (0, 1)] for p in range(16)] for b in range(64)],
                       dtype=np.float32)
        assert np.array_equal(got, ref)


def test_philox_two_implementations_agree_on_a_million_counters(oracle):
    """2^20 counters (round, b, pos), two words each: the HIP generator against the oracle's (which is itself
    pinned against rocRAND's engine on the CPU)."""
    import ctypes as C
    B, npos = 16384, 32                                         # B * npos = 2^19 counters per round value
    cfg = binding.make_cfg(V=8, d=8, n=1, B=B, gamma=npos - 1, h=1, w_dtype=0, seed=0xC0FFEE1234567)
    out = torch.zeros((B, npos, 2), dtype=torch.float32, device=DEV)
    lib = oracle.lib()
    for rnd in (3, (1 << 33) + 9):
        binding.tabed_philox_uniforms(cfg, rnd, out)
        got = out.cpu().numpy()
        ref = np.empty((B, npos, 2), np.float32)
        for b in range(B):
            for p in range(npos):
                ref[b, p, 0] = lib.oracle_uniform(cfg.seed, rnd, b, p, 0)
                ref[b, p, 1] = lib.oracle_uniform(cfg.seed, rnd, b, p, 1)
        assert np.array_equal(got, ref), rnd


# ------------------------------------------------------------------ the paper-scale tiny configuration, 64 rounds
@pytest.mark.parametrize("mode", ["greedy", "one"])
def test_tiny_64_rounds_state_carried(oracle, mode):
    _say(f"tiny {mode}")
    tally = harness.run_rounds(oracle, TINY, TINY.rounds, synth.make_temperature(TINY, mode))
    _say(tally)
    assert tally.flagged_divergences <= 2


# ------------------------------------------------------------------ shapes that span several tiles with ragged tails
SHAPES = [
    # V,     d,   n, B, gamma, h, w_dtype, temperature
    (1000,   64,  2, 3, 3,     4, 1, "one"),        # bf16, V not a multiple of 64
    (4099,   72,  3, 5, 4,     5, 1, "mixed07"),    # V % 4 != 0: scalar loads; d not a multiple of 64
    (8200,   128, 4, 2, 2,     3, 1, "greedy"),     # two full 4096-chunks and an 8-element tail
    (33,     8,   1, 1, 1,     1, 1, "one"),        # one draft, one token
    (257,    40,  16, 2, 2,    2, 0, "one"),        # maximum number of drafts, fp32 storage
    (5000,   64,  5, 70, 2,    3, 1, "mixed07"),    # more rows than one 64-row MFMA tile
    (1,      8,   2, 2, 2,     2, 0, "one"),        # single-token vocabulary
    # shapes that take the W-streaming LM-head kernel (bf16, n*B <= 64, d in {512, 768, 896, 1024})
    (1000,   512, 2, 3, 2,     4, 1, "one"),        # one 32-row block of M, ragged last vocabulary tile
    (2084,   896, 4, 8, 2,     3, 1, "mixed07"),    # n*B = 32, tile count not a multiple of 4
    (4099,  1024, 4, 16, 2,    3, 1, "one"),        # n*B = 64, V % 4 != 0
    (40000,  768, 4, 16, 1,    3, 1, "one"),        # more tile groups than workgroups: persistent loop runs twice
    (33000,  768, 3, 11, 2,    3, 1, "greedy"),     # n*B = 33: second row block almost empty
    (70004,  64,  4, 3, 2,     3, 1, "mixed07"),    # more than 2048 softmax tiles: 20 tiles per sampler thread
    (200003, 64,  2, 2, 1,     2, 1, "mixed07"),    # beyond 163840: 32 tiles per sampler thread, two-pass sampler
    (700,    16,  16, 2, 32,   300, 1, "mixed07"),  # maximum block length and draft count, window longer than the run
    # larger hidden sizes with n*B <= 64: the K-chunked streaming LM head
    (2100,  1024, 4, 16, 2,    3, 1, "one"),        # two chunks of 512, two row blocks
    (40000, 1536, 2, 5, 1,     3, 1, "mixed07"),    # two chunks of 768, one row block, persistent loop twice
    (1000,  2048, 4, 12, 2,    3, 1, "one"),        # four chunks of 512, ragged last tile
    (700,   1792, 3, 3, 1,     2, 1, "greedy"),     # two chunks of 896
    # shapes that take the many-rows LM-head kernel (bf16, n*B > 64, d % 64 == 0)
    (4099,   256, 8, 40, 2,    3, 1, "one"),        # 320 rows: two row blocks, V % 4 != 0 (element-wise epilogue)
    (3000,   128, 8, 70, 1,    3, 1, "mixed07"),    # 560 rows: three row blocks, ragged last vocabulary block
    (900,    64,  8, 20, 1,    2, 1, "one"),        # 160 rows, one k-block in all
    (262144, 64,  2, 2, 1,     2, 1, "mixed07"),    # the largest vocabulary the library takes
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: f"V{s[0]}d{s[1]}n{s[2]}B{s[3]}g{s[4]}")
def test_shapes_and_edges(oracle, shape):
    V, d, n, B, gamma, h, w_dtype, mode = shape
    _say(f"shape {shape}")
    wl = synth.scaled(SERVING, V=V, d=d, n=n, B=B, gamma=gamma, h=h, w_dtype=w_dtype, cfg_id=40 + V % 7)
    tally = harness.run_rounds(oracle, wl, 6, synth.make_temperature(wl, mode))
    _say(tally)
    assert tally.flagged_divergences <= max(2, tally.decisions // 50)


def test_static_policy_and_other_tau(oracle):
    wl = synth.scaled(SERVING, V=2048, d=64, B=4, cfg_id=51)
    t = harness.run_rounds(oracle, wl, 4, synth.make_temperature(wl, "one"), policy=1)
    assert t.max_w_err == 0.0


# ------------------------------------------------------------------ total variation distance and the two-draft grid policy
@pytest.mark.parametrize("policy,distance,n", [(0, 1, 4), (2, 0, 2), (2, 1, 2), (1, 1, 3), (3, 0, 5), (2, 2, 2), (0, 2, 4)],
                         ids=["tvd", "grid-kl", "grid-tvd", "static-tvd", "random-weights", "grid-hard", "hard"])
def test_distance_and_policy_variants(oracle, policy, distance, n):
    for V, d, B, mode in ((4100, 64, 5, "mixed07"), (4099, 72, 3, "one"), (32000, 768, 4, "one")):
        wl = synth.scaled(SERVING, V=V, d=d, n=n, B=B, gamma=3, h=5, cfg_id=70 + policy * 2 + distance)
        _say(f"variant policy={policy} distance={distance} V={V}")
        tally = harness.run_rounds(oracle, wl, 5, synth.make_temperature(wl, mode), policy=policy, distance=distance)
        _say(tally)
        assert tally.flagged_divergences <= max(2, tally.decisions // 50)


@pytest.mark.parametrize("policy,distance,n,h,mode", [(0, 0, 4, 8, "one"), (0, 0, 3, 5, "mixed07"), (2, 1, 2, 0, "one"),
                                                        (0, 0, 4, 0, "greedy"), (3, 0, 16, 4, "mixed07"), (2, 2, 2, 6, "mixed07"),
                                                        (2, 2, 2, 0, "greedy")],
                         ids=["softmax", "mixed-rows", "grid-tvd-all", "greedy-all", "random-16-drafts", "grid-hard-mixed",
                              "grid-hard-greedy"])
def test_verify_with_fused_window_update(oracle, policy, distance, n, h, mode):
    """tabed_verify given the window pointers must leave the same window and next weights as the separate
    tabed_update_weights call the oracle models."""
    for V, d, B in ((4100, 64, 5), (32000, 768, 16)):
        wl = synth.scaled(SERVING, V=V, d=d, n=n, B=B, gamma=4, h=h, cfg_id=90 + policy + distance)
        tally = harness.run_rounds(oracle, wl, 8, synth.make_temperature(wl, mode), policy=policy, distance=distance,
                                   fused=True)
        _say(tally)
        assert tally.flagged_divergences <= max(2, tally.decisions // 50)


def test_window_all(oracle):
    """h = 0: the paper's default window (all verified positions since the start)."""
    for policy, n in ((0, 4), (2, 2)):
        wl = synth.scaled(SERVING, V=4100, d=64, n=n, B=6, gamma=4, h=0, cfg_id=80 + policy)
        tally = harness.run_rounds(oracle, wl, 12, synth.make_temperature(wl, "one"), policy=policy)
        _say(tally)
        assert tally.flagged_divergences <= 1


# ------------------------------------------------------------------ explicit uniforms, including the edges of [0,1)
def test_explicit_uniform_edges(oracle):
    wl = synth.scaled(SERVING, V=3000, d=64, n=3, B=8, gamma=3, h=4, cfg_id=52)
    edge = np.array([0.0, 1 - 2.0 ** -24, 0.5, 0.25, 2.0 ** -24, 0.75, 0.999, 0.001], np.float32)

    def uniforms(rnd):
        return dict(u_draft=np.tile(np.roll(edge, rnd)[:, None], (1, wl.gamma)),
                    u_acc=np.tile(np.roll(edge, rnd + 3)[:, None], (1, wl.gamma)),
                    u_res=np.roll(edge, rnd + 5).copy())
    tally = harness.run_rounds(oracle, wl, 8, synth.make_temperature(wl, "one"), uniforms=uniforms)
    _say(tally)


def test_identical_draft_and_target_always_accepts(oracle):
    """n = 1 and target logits equal to the draft's: p == q, every token accepted, bonus token emitted."""
    wl = synth.scaled(SERVING, V=2000, d=64, n=1, B=4, gamma=4, h=4, cfg_id=53, target="draft0", sigma=0.0)
    W = synth.make_lm_head(wl)
    gpu = harness.GpuSide(wl)
    H, target = synth.make_round(wl, W, 0)
    g = gpu.round(0, harness.to_dev_store(W, wl.w_dtype), H, target, synth.make_temperature(wl, "one"))
    # the recipe's matmul and the kernel's differ in the last bits, so p/q is 1 +- 1e-6: accepted unless u ~ 1
    assert np.all(g["accept_len"] == wl.gamma)
    assert np.all(g["out_tokens"] >= 0)
    assert np.all(g["dev"] < 1e-6)


def test_out_of_range_draft_token_is_rejected_not_dereferenced(oracle):
    wl = synth.scaled(SERVING, V=1500, d=64, n=2, B=3, gamma=3, h=4, cfg_id=54)
    W = synth.make_lm_head(wl)
    gpu = harness.GpuSide(wl)
    temp = synth.make_temperature(wl, "one")
    H, target = synth.make_round(wl, W, 0)
    gpu.round(0, harness.to_dev_store(W, wl.w_dtype), H, target, temp)
    buf = gpu.buf
    buf.draft_tokens[1, 0] = wl.V + 12345
    buf.draft_tokens[2, 1] = -7
    buf.verify(0, torch.from_numpy(target).to(DEV), torch.from_numpy(temp).to(DEV))
    torch.cuda.synchronize()
    assert buf.accept_len[1].item() == 0 and buf.verify_flags[1, 0].item() & binding.FLAG_DEGENERATE
    assert buf.accept_len[2].item() <= 1
    assert 0 <= buf.out_tokens[1, 0].item() < wl.V


def test_hard_label_near_tie_of_a_mixture_is_flagged(oracle):
    """Two-draft grid with hard labels, hand-made logits handed to tabed_verify: a mixture whose two largest entries
    tie (in one 4096-wide chunk for sequence 0, across chunks for sequence 1) flags the labelled position on both
    sides, not the positions after the rejection; distances and tokens agree exactly."""
    V, gamma, B = 9000, 4, 2
    wl = synth.scaled(SERVING, V=V, d=64, n=2, B=B, gamma=gamma, h=4, cfg_id=55)
    gpu = harness.GpuSide(wl, policy=2, distance=2)
    W = synth.make_lm_head(wl)
    H, target0 = synth.make_round(wl, W, 0)
    temp = np.array([0.0, 1.0], np.float32)                    # sequence 0 greedy, sequence 1 sampling
    gpu.round(0, harness.to_dev_store(W, wl.w_dtype), H, target0, temp)
    buf = gpu.buf
    logq = np.full((gamma, B, 2, V), -3.0, np.float32)
    logq[:, :, :, 3] = 1.0                                     # both drafts: mode on token 3
    logq[1, 0, :, 7] = 1.0                                     # position 1: a second token ties with it (same chunk)
    logq[1, 1, :, 5000] = 1.0                                  # ... (another chunk)
    logq[3, :, :, 7] = 1.0                                     # position 3 comes after the rejection
    logp = np.full((B, gamma + 1, V), -3.0, np.float32)
    logp[:, 0, 3] = logp[:, 1, 3] = 4.0                        # the target agrees at 0 and 1, wants token 5 at 2
    logp[:, 2, 5] = 4.0
    tok = np.full((B, gamma), 3, np.int32)
    q_y = np.array([[oracle.softmax(logq[i, b, 0], 1.0)[0][3] for i in range(gamma)] for b in range(B)], np.float32)
    lse = np.log(np.exp(logq.astype(np.float64)).sum(axis=-1))
    u_acc = np.array([[0.01, 0.01, 0.9, 0.9]] * B, np.float32)
    u_res = np.array([0.5, 0.5], np.float32)
    buf.draft_logits.copy_(torch.from_numpy(logq))
    buf.draft_lse.copy_(torch.from_numpy(lse))
    buf.draft_tokens.copy_(torch.from_numpy(tok))
    buf.draft_q.copy_(torch.from_numpy(q_y))
    dev_t = lambda a: torch.from_numpy(a).to(DEV)
    buf.verify(1, dev_t(logp), dev_t(temp), dev_t(u_acc), dev_t(u_res))
    torch.cuda.synchronize()
    weights = buf.weights.cpu().numpy()
    o = oracle.verify(V=V, n=2, B=B, gamma=gamma, distance=2, seed=0, rnd=1, n_cand=oracle.GRID_CANDIDATES,
                      target_logits=logp, draft_logits=logq, draft_tokens=tok, draft_q=q_y, weights=weights,
                      temperature=temp, u_acc=u_acc, u_res=u_res)
    SM = binding.FLAG_SAMPLE_MARGIN
    g_flags = buf.verify_flags.cpu().numpy()
    assert np.array_equal(buf.accept_len.cpu().numpy(), o["accept_len"]) and np.all(o["accept_len"] == 2)
    assert np.array_equal(buf.out_tokens.cpu().numpy(), o["out_tokens"])
    assert np.array_equal(buf.dev.cpu().numpy(), o["dev"])
    for b in range(B):
        for side in (g_flags, o["flags"]):
            assert side[b, 1] & SM and not side[b, 0] & SM and not side[b, 3] & SM, (b, side[b])


def test_grid_policy_with_nearly_equal_candidates(oracle):
    """Two drafts with a tiny hidden size are almost the same distribution, so the 11 candidate mixtures are too and
    their window sums differ in the seventh digit: the arg-min may then legitimately differ between the two sides.
    The harness accepts that only after checking the oracle-side sums of the two candidates against the tolerance
    of the distances (a case found by a wider random sweep)."""
    wl = synth.scaled(SERVING, V=8053, d=5, n=2, B=20, gamma=6, h=2, w_dtype=0, cfg_id=3035, target="independent", sigma=1.0)
    tally = harness.run_rounds(oracle, wl, 3, synth.make_temperature(wl, "one"), seed=35, policy=2, distance=0)
    _say(tally)
    assert tally.flagged_divergences <= 3


# ------------------------------------------------------------------ the lossless property, on the GPU path alone
@pytest.mark.parametrize("width", [1, 2, 3], ids=["chain", "tree2", "tree3"])
def test_emitted_tokens_follow_the_target_distribution(width):
    """Speculative sampling is lossless (Sec. 3 item 3): whatever the drafts propose, the first token a round emits
    is distributed as p_0, and so is the token at position 1 when the round gets that far -- also with a token tree,
    whose extra candidates only raise the chance of keeping a drafted token.  No oracle here: 64 sequences with the
    same inputs and their own Philox streams, 400 rounds, chi-square of the emitted tokens against softmax of the
    target logits (V = 12; the drafts are deliberately far from the target so that every branch of the rule runs)."""
    from scipy.stats import chi2
    V, d, n, B, gamma, R = 12, 16, 2, 64, 3, 400
    cfg = binding.make_cfg(V=V, d=d, n=n, B=B, gamma=gamma, h=4, w_dtype=1, policy=1, seed=1234)
    buf = binding.RoundBuffers(cfg, DEV)
    S = width - 1
    rng = np.random.default_rng(77)
    W = harness.to_dev_store(synth.bf16_bits(rng.standard_normal((V, d), dtype=np.float32) * 0.4), 1)
    H1 = rng.standard_normal((gamma, n, d), dtype=np.float32)
    Hs = [harness.to_dev_store(synth.bf16_bits(np.broadcast_to(H1[i], (B, n, d)).copy()), 1) for i in range(gamma)]
    t1 = (rng.standard_normal((gamma + 1, V)) * 1.2).astype(np.float32)
    target = torch.from_numpy(np.broadcast_to(t1, (B, gamma + 1, V)).copy()).to(DEV)
    l1 = (rng.standard_normal((gamma, max(S, 1), V)) * 1.2).astype(np.float32)
    leaves = torch.from_numpy(np.broadcast_to(l1, (B, gamma, max(S, 1), V)).copy()).to(DEV)
    temp = torch.ones(B, device=DEV)
    sib_tok = torch.zeros((B, gamma, max(S, 1)), dtype=torch.int32, device=DEV)
    sib_q = torch.zeros((B, gamma, max(S, 1)), dtype=torch.float32, device=DEV)
    sib_fl = torch.zeros((B, gamma, max(S, 1)), dtype=torch.uint8, device=DEV)
    leaf = torch.zeros(B, dtype=torch.int32, device=DEV)
    n_out = torch.zeros(B, dtype=torch.int32, device=DEV)
    buf.update_weights(True)
    first = np.zeros(V)
    second = np.zeros(V)
    after_leaf = np.zeros((gamma, max(S, 1), V))
    kept = 0
    for rnd in range(R):
        for pos in range(gamma):
            buf.draft_step(rnd, pos, W, Hs[pos], temp)
            if S:
                binding.tabed_draft_siblings(cfg, buf.ws, rnd, pos, width, buf.draft_logits, buf.draft_tokens, buf.weights, temp,
                                             sib_tok, sib_q, sib_fl)
        if S:
            binding.tabed_verify_tree(cfg, buf.ws, rnd, width, target, leaves, buf.draft_logits, buf.draft_lse, buf.draft_tokens,
                                      buf.draft_q, sib_tok, sib_q, buf.weights, temp, buf.accept_len, buf.out_tokens, buf.dev,
                                      buf.n_valid, buf.verify_flags, leaf, n_out)
        else:
            buf.verify(rnd, target, temp)
        torch.cuda.synchronize()
        out, k = buf.out_tokens.cpu().numpy(), buf.accept_len.cpu().numpy()
        lf = leaf.cpu().numpy() if S else np.zeros(B, np.int32)
        first += np.bincount(out[:, 0], minlength=V)
        # position 1 is reached when the token at 0 was kept as the TRUNK token (a leaf ends the round's drafted part)
        reached = (k >= 1)
        second += np.bincount(out[reached, 1], minlength=V)
        kept += int(k.sum())
        for b in np.nonzero(lf > 0)[0]:                     # the token after an accepted leaf follows that leaf's row
            after_leaf[k[b], lf[b] - 1, out[b, k[b] + 1]] += 1

    def check(counts, logits, what):
        p = np.exp(logits.astype(np.float64) - logits.max())
        p /= p.sum()
        N = counts.sum()
        assert N > 1500, (what, N)
        rare = N * p < 8                                    # bins too small for the chi-square approximation: one bin
        obs = np.append(counts[~rare], counts[rare].sum())
        exp = np.append(N * p[~rare], N * p[rare].sum())
        obs, exp = obs[exp > 0], exp[exp > 0]
        stat = float(((obs - exp) ** 2 / exp).sum())
        assert stat < chi2.ppf(1 - 1e-6, len(exp) - 1), (what, stat, obs, exp)

    check(first, t1[0], "first emitted token")
    check(second, t1[1], "token at position 1")
    assert 0 < kept < R * B * gamma                         # both accepting and rejecting happened
    if S:
        tot = after_leaf.sum(axis=-1)
        i, s_ = np.unravel_index(np.argmax(tot), tot.shape)
        check(after_leaf[i, s_], l1[i, s_], f"token after leaf {s_ + 1} of position {i}")


# ------------------------------------------------------------------ the window / weights kernel alone
def test_update_weights_alone_matches_oracle_bitwise_state(oracle):
    rng = np.random.default_rng(60)
    B, n, gamma, h = 37, 7, 5, 6
    cfg = binding.make_cfg(V=8, d=8, n=n, B=B, gamma=gamma, h=h, w_dtype=0, tau_w=0.5, eps=1e-6)
    ws = binding.new_workspace(cfg)
    ring = torch.zeros((B, h, n), device=DEV); head = torch.zeros(B, dtype=torch.int32, device=DEV)
    count = torch.zeros(B, dtype=torch.int32, device=DEV); w = torch.zeros((B, n), device=DEV)
    o_ring = np.zeros((B, h, n), np.float32); o_head = np.zeros(B, np.int32); o_count = np.zeros(B, np.int32)
    for step in range(12):
        dev = (rng.random((B, gamma, n)) * (10.0 ** rng.uniform(-4, 0.5, (B, 1, 1)))).astype(np.float32)
        nv = rng.integers(1, gamma + 1, B).astype(np.int32)
        if step == 0:
            binding.tabed_update_weights(cfg, ws, 0, None, None, ring, head, count, w)
            ow = oracle.update_weights(n=n, B=B, gamma=gamma, h=h, policy=0, tau_w=0.5, eps=1e-6, dev=None,
                                       n_valid=None, ring=o_ring, ring_head=o_head, ring_count=o_count)
        else:
            binding.tabed_update_weights(cfg, ws, step, torch.from_numpy(dev).to(DEV), torch.from_numpy(nv).to(DEV),
                                         ring, head, count, w)
            ow = oracle.update_weights(n=n, B=B, gamma=gamma, h=h, policy=0, tau_w=0.5, eps=1e-6, dev=dev,
                                       n_valid=nv, ring=o_ring, ring_head=o_head, ring_count=o_count)
        torch.cuda.synchronize()
        assert np.array_equal(ring.cpu().numpy(), o_ring)
        assert np.array_equal(head.cpu().numpy(), o_head) and np.array_equal(count.cpu().numpy(), o_count)
        np.testing.assert_allclose(w.cpu().numpy(), ow, rtol=1e-6, atol=1e-30)


# ------------------------------------------------------------------ determinism: same call, same bits
def test_two_runs_are_bitwise_identical(oracle):
    wl = synth.scaled(SERVING, V=32000, B=4, cfg_id=55)
    W = synth.make_lm_head(wl)
    W_t = harness.to_dev_store(W, wl.w_dtype)
    temp = synth.make_temperature(wl, "mixed07")
    H, target = synth.make_round(wl, W, 0)
    outs = []
    for _ in range(2):
        gpu = harness.GpuSide(wl)
        outs.append(gpu.round(0, W_t, H, target, temp))
    for key in outs[0]:
        assert np.array_equal(outs[0][key], outs[1][key]), key


# ------------------------------------------------------------------ full size, in the launch configuration bench.py times
def test_serving_full_size_rounds(oracle):
    _say("serving full size")
    tally = harness.run_rounds(oracle, SERVING, 24, synth.make_temperature(SERVING))     # the h = 8 window wraps many times
    _say(tally)
    assert tally.flagged_divergences <= 2


def test_llava_full_size_greedy_and_sampling(oracle):
    wl = synth.WORKLOADS["llava"]
    for mode in ("greedy", "one"):
        _say(f"llava {mode}")
        tally = harness.run_rounds(oracle, wl, 16, synth.make_temperature(wl, mode))
        _say(tally)
        assert tally.flagged_divergences <= 1


def test_lvlm_full_size(oracle):
    """V=152064, d=896, n=4, B=8, gamma=7, h=16 with the matching draft switching: the large-vocabulary LVLM workload."""
    wl = synth.WORKLOADS["lvlm"]
    _say("lvlm full size")
    tally = harness.run_rounds(oracle, wl, 2, synth.make_temperature(wl))
    _say(tally)
    assert tally.flagged_divergences <= 3


def test_stress_shape_fewer_sequences(oracle):
    """The stress vocabulary, hidden size, draft count and temperature mix (V=128256, d=2048, n=8, greedy and
    T=0.7 rows, heavy-tailed target noise) on 12 sequences and 2 positions: 96 rows through the many-rows LM head,
    every sequence compared."""
    wl = synth.scaled(synth.WORKLOADS["stress"], B=12, gamma=2, cfg_id=95)
    _say("stress shape, 12 sequences")
    tally = harness.run_rounds(oracle, wl, 2, synth.make_temperature(wl))
    _say(tally)
    assert tally.flagged_divergences <= 3


def test_stress_full_size_against_oracle_on_a_subset(oracle):
    """The stress workload at its real size (V=128256, d=2048, n=8, B=64, gamma=5, h=16: 512 rows through the
    many-rows LM head, two row blocks): the GPU runs all 64 sequences, the oracle a subset of six of them
    (greedy and T=0.7 rows, first / middle / last row block), element by element, state carried over two rounds."""
    wl = synth.WORKLOADS["stress"]
    rows = [0, 1, 30, 33, 62, 63]
    _say("stress full size, oracle on sequences " + str(rows))
    tally = harness.run_rounds(oracle, wl, 2, synth.make_temperature(wl), rows=rows)
    _say(tally)
    assert tally.flagged_divergences <= 2


def test_lvlm_full_size_across_a_draft_switch(oracle):
    """The large-vocabulary workload at full size, rounds 60..73: the draft the target follows changes at round
    64, the 16-entry window wraps, and on both sides the largest weight moves from the old matching draft to
    the new one."""
    wl = synth.WORKLOADS["lvlm"]
    rows = [0, 3, 7]
    seen = {}

    def on_round(rnd, g, o):
        seen[rnd] = (np.argmax(g["weights"], axis=1), np.argmax(o["weights"], axis=1), o["n_valid"].copy())
        _say(f"  round {rnd}: matching draft {synth.matching_draft(wl, rnd)} argmax w gpu {seen[rnd][0]} oracle {seen[rnd][1]} "
             f"n_valid {seen[rnd][2]}")

    _say("lvlm full size across the switch at round 64")
    tally = harness.run_rounds(oracle, wl, 14, synth.make_temperature(wl), start_round=60, rows=rows, on_round=on_round)
    _say(tally)
    assert tally.flagged_divergences <= 3
    old, new = synth.matching_draft(wl, 63), synth.matching_draft(wl, 64)
    assert old != new
    # weights used in round 63 were learned from rounds 60..62 (old draft); the weights used in round 73 from a
    # window that holds only positions verified after the switch (>= 16 of them in rounds 64..72)
    assert np.all(seen[63][0] == old) and np.all(seen[63][1] == old)
    assert np.all(sum(seen[r][2] for r in range(64, 73)) >= wl.h)       # every sequence's window has wrapped
    assert np.all(seen[73][0] == new) and np.all(seen[73][1] == new)


def test_lvlm_recipe_70_rounds_reduced_vocabulary(oracle):
    """The same recipe (d=896, n=4, B=8, gamma=7, h=16, switch every 64 rounds) at a reduced vocabulary, all
    sequences, state carried from round 0 across the switch: window wrap and adaptation through the same kernels."""
    wl = synth.scaled(synth.WORKLOADS["lvlm"], V=4100)
    last = {}

    def on_round(rnd, g, o):
        last[rnd] = (np.argmax(g["weights"], axis=1), np.argmax(o["weights"], axis=1))

    tally = harness.run_rounds(oracle, wl, 72, synth.make_temperature(wl), on_round=on_round)
    _say(tally)
    assert tally.flagged_divergences <= 4
    assert np.all(last[63][0] == 0) and np.all(last[63][1] == 0)
    assert np.all(last[71][0] == 1) and np.all(last[71][1] == 1)


# ------------------------------------------------------------------ token tree (Sec. 6.1)
TREE_CASES = [
    # V,     d,   n, B, gamma, h, w_dtype, temperature, width, fused window update, explicit uniforms
    (1000,   64,  2, 3, 3,     4, 0, "one",     2, False, False),
    (4099,   72,  3, 5, 4,     5, 1, "mixed07", 3, False, False),    # V % 4 != 0, greedy and sampling rows
    (8200,   128, 4, 6, 2,     3, 1, "greedy",  3, False, False),
    (40,     16,  2, 24, 3,    3, 1, "greedy",  3, False, False),    # tiny vocabulary: greedy siblings do get accepted
    (5000,   64,  5, 9, 2,     3, 1, "mixed07", 2, True,  True),
    (32000,  768, 4, 16, 5,    8, 1, "one",     2, False, False),    # the serving shape
    (32000,  768, 4, 16, 5,    8, 1, "one",     3, True,  False),
    (152064, 896, 4, 2, 2,     16, 1, "mixed07", 3, False, False),   # large vocabulary: several segments per thread
]


@pytest.mark.parametrize("case", TREE_CASES, ids=lambda c: f"V{c[0]}n{c[2]}B{c[3]}w{c[8]}{c[7]}")
def test_token_tree_matches_oracle(oracle, case):
    V, d, n, B, gamma, h, w_dtype, mode, width, fused, explicit = case
    _say(f"token tree {case}")
    wl = synth.scaled(SERVING, V=V, d=d, n=n, B=B, gamma=gamma, h=h, w_dtype=w_dtype, cfg_id=130 + V % 11)
    # the 40-token case runs with static weights: its distances are tiny, and 1/e would amplify their rounding
    tally = harness.run_rounds_tree(oracle, wl, 5, synth.make_temperature(wl, mode), width, fused=fused,
                                    explicit_uniforms=explicit, policy=1 if V < 100 else 0)
    _say(f"{tally} leaves={tally.leaves} emitted={tally.emitted}")
    assert tally.flagged_divergences <= max(2, tally.decisions // 50)
    assert tally.leaves > 0 or mode == "greedy" or B * 5 < 20      # sibling acceptances are exercised


def test_token_tree_of_width_one_is_the_chain(oracle):
    """tabed_verify_tree with tree_width = 1 leaves exactly what tabed_verify leaves, plus leaf = 0 and n_out = k + 1."""
    wl = synth.scaled(SERVING, V=8200, d=128, B=6, gamma=3, cfg_id=141)
    W = synth.make_lm_head(wl)
    temp = synth.make_temperature(wl, "mixed07")
    H, target = synth.make_round(wl, W, 0)
    gpu = harness.GpuSide(wl)
    ref = gpu.round(0, harness.to_dev_store(W, wl.w_dtype), H, target, temp)
    buf = gpu.buf
    leaf = torch.full((wl.B,), -7, dtype=torch.int32, device=DEV)
    n_out = torch.full((wl.B,), -7, dtype=torch.int32, device=DEV)
    for t in (buf.accept_len, buf.out_tokens, buf.n_valid):
        t.fill_(-9)
    buf.dev.fill_(-1.0)
    binding.tabed_verify_tree(gpu.cfg, buf.ws, 0, 1, torch.from_numpy(target).to(DEV), None, buf.draft_logits, buf.draft_lse,
                              buf.draft_tokens, buf.draft_q, None, None, buf.weights, torch.from_numpy(temp).to(DEV),
                              buf.accept_len, buf.out_tokens, buf.dev, buf.n_valid, buf.verify_flags, leaf, n_out)
    torch.cuda.synchronize()
    for key, tens in (("accept_len", buf.accept_len), ("out_tokens", buf.out_tokens), ("dev", buf.dev),
                      ("n_valid", buf.n_valid), ("flags", buf.verify_flags)):
        assert np.array_equal(tens.cpu().numpy(), ref[key]), key
    assert np.all(leaf.cpu().numpy() == 0) and np.array_equal(n_out.cpu().numpy(), ref["accept_len"] + 1)


def test_hip_graph_replay_matches_eager_bitwise(oracle):
    """bench.py replays captured rounds: a captured sequence of the C-ABI calls must give, on every replay,
    exactly what the same calls give when issued eagerly from the same state."""
    import ctypes as C
    wl = synth.scaled(SERVING, V=32000, B=8, gamma=3, cfg_id=97)
    W = synth.make_lm_head(wl)
    W_t = harness.to_dev_store(W, wl.w_dtype)
    temp_t = torch.from_numpy(synth.make_temperature(wl, "mixed07")).to(DEV)
    rounds = [synth.make_round(wl, W, r) for r in range(2)]
    H_t = [[harness.to_dev_store(H[pos], wl.w_dtype) for pos in range(wl.gamma)] for H, _ in rounds]
    T_t = [torch.from_numpy(t).to(DEV) for _, t in rounds]
    cfg = harness.cfg_of(wl)
    buf = binding.RoundBuffers(cfg, DEV)
    keys = ("weights", "ring", "ring_head", "ring_count", "draft_tokens", "draft_q", "draft_lse", "accept_len",
            "out_tokens", "dev", "n_valid", "verify_flags", "draft_flags")

    def reset():
        for k in ("weights", "ring", "ring_head", "ring_count", "dev", "n_valid"):
            getattr(buf, k).zero_()

    def two_rounds(stream=None):
        buf.update_weights(True, stream=stream)
        for r in range(2):
            for pos in range(wl.gamma):
                buf.draft_step(r, pos, W_t, H_t[r][pos], temp_t, stream=stream)
            buf.verify(r, T_t[r], temp_t, stream=stream, fused_update=True)

    def snapshot():
        torch.cuda.synchronize()
        return {k: getattr(buf, k).clone() for k in keys}

    reset()
    two_rounds()
    eager = snapshot()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        reset()
        two_rounds(side)                      # once on the side stream before capture
        side.synchronize()
        reset()
        with torch.cuda.graph(graph, stream=side):
            two_rounds(side)
    torch.cuda.synchronize()
    for replay in range(3):
        reset()
        scratch = torch.randn(1 << 20, device=DEV).sum()       # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for k in keys:
            assert torch.equal(got[k], eager[k]), (replay, k)
        del scratch


def test_soak_two_thousand_rounds_twice_bitwise(oracle):
    """The cross-workgroup hand-overs (greedy arg-max merge, corrected-token sampler, fused window update) under
    sustained load: 2000 serving-shape rounds with greedy and sampling rows, window state carried, run twice from
    the same state -- every round's tokens, accept lengths, distances and weights must be bit-identical.  A stale
    partial result read by a finishing workgroup would show up as a difference; the comparison names the first
    round that differs."""
    wl = synth.scaled(SERVING, cfg_id=98)
    rounds, pool = 2000, 6
    W = synth.make_lm_head(wl)
    W_t = harness.to_dev_store(W, wl.w_dtype)
    temp_t = torch.from_numpy(synth.make_temperature(wl, "mixed07")).to(DEV)
    inputs = [synth.make_round(wl, W, r) for r in range(pool)]
    H_t = [[harness.to_dev_store(H[pos], wl.w_dtype) for pos in range(wl.gamma)] for H, _ in inputs]
    T_t = [torch.from_numpy(t).to(DEV) for _, t in inputs]
    cfg = harness.cfg_of(wl, seed=5)
    logs = []
    for run in range(2):
        buf = binding.RoundBuffers(cfg, DEV)
        log_tok = torch.zeros((rounds, wl.B, wl.gamma + 1), dtype=torch.int32, device=DEV)
        log_dtok = torch.zeros((rounds, wl.B, wl.gamma), dtype=torch.int32, device=DEV)
        log_dev = torch.zeros((rounds, wl.B, wl.gamma, wl.n), dtype=torch.float32, device=DEV)
        log_w = torch.zeros((rounds, wl.B, wl.n), dtype=torch.float32, device=DEV)
        buf.update_weights(True)
        for r in range(rounds):
            log_w[r].copy_(buf.weights)
            for pos in range(wl.gamma):
                buf.draft_step(r, pos, W_t, H_t[r % pool][pos], temp_t)
            buf.verify(r, T_t[r % pool], temp_t, fused_update=True)
            log_tok[r].copy_(buf.out_tokens)
            log_dtok[r].copy_(buf.draft_tokens)
            log_dev[r].copy_(buf.dev)
            if r % 500 == 499:
                torch.cuda.synchronize()
                _say(f"  soak run {run}: {r + 1} rounds")
        torch.cuda.synchronize()
        logs.append((log_tok, log_dtok, log_dev, log_w))
    for name, a, b in zip(("out_tokens", "draft_tokens", "dev", "weights"), logs[0], logs[1]):
        same = (a.view(torch.int32) == b.view(torch.int32)).flatten(1).all(dim=1)
        if not bool(same.all()):
            first = int((~same).nonzero()[0])
            raise AssertionError(f"{name} differs between the two runs from round {first} on")
    assert int((logs[0][0][:, :, 0] >= 0).sum()) == rounds * wl.B          # every round emitted a token per sequence


def test_seeded_sweep_of_small_shapes(oracle):
    """Twenty seeded random configurations (vocabulary, hidden size, drafts, sequences, block length, window,
    storage type, temperature mix, policy, distance, fused or separate window update)."""
    rng = np.random.default_rng(2024)
    for case in range(20):
        w_dtype = int(rng.integers(0, 2))
        d = int(rng.choice([8, 24, 64, 72, 128, 256, 512] if w_dtype else [5, 8, 33, 64]))
        policy = int(rng.choice([0, 0, 0, 1, 2, 3]))
        n = 2 if policy == 2 else int(rng.integers(1, 10))
        distance = int(rng.integers(0, 3))
        B = int(rng.integers(1, 23))
        wl = synth.scaled(SERVING, V=int(rng.integers(1, 9000)), d=d, n=n, B=B, gamma=int(rng.integers(1, 7)),
                          h=int(rng.integers(0, 9)), w_dtype=w_dtype, cfg_id=200 + case,
                          target=str(rng.choice(["per_seq_sigma", "independent", "student_t"])), sigma=1.0)
        mode = str(rng.choice(["one", "greedy", "mixed07"]))
        fused = bool(rng.integers(0, 2))
        _say(f"case {case}: V={wl.V} d={d} n={n} B={B} gamma={wl.gamma} h={wl.h} w_dtype={w_dtype} {mode} "
             f"policy={policy} distance={distance} fused={fused} target={wl.target}")
        tally = harness.run_rounds(oracle, wl, 4, synth.make_temperature(wl, mode), seed=case, policy=policy,
                                   distance=distance, fused=fused)
        assert tally.flagged_divergences <= max(2, tally.decisions // 25), tally
