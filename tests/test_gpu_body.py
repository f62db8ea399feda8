"""GPU parity of the draft-model body (tabed_draft_body_step) against the fp64 oracle with the same storage points.

The two sides differ by the accumulation precision of the projections (fp32 MFMA against fp64) and by fp32
reductions in the norms and in attention.  A value that lands within that error of a bf16 rounding boundary comes
out one bf16 step apart, and such a flip is a real 2^-8 perturbation of one input of the following layers, where it
causes further flips: with depth the two results drift apart until they differ by about the rounding noise of the
format itself (measured: relative RMS difference 2.7e-4 after one layer, 6e-4 after two, 2.4e-3 after twelve, 3.7e-3
= one bf16 step after sixteen), and no further.  The bars, from that:
  * at any depth: relative RMS difference of a tensor at most 2^-7 (two bf16 steps), no entry further than 2^-6 of
    its row's largest magnitude;
  * up to two layers, where the flips are still few: at most 1 % of the entries more than one bf16 step apart
    (2^-7 relative, with an absolute floor for entries near zero);
cache entries written by the step obey the same bars, every other cache entry is untouched, positions advance
exactly.  Each step is judged from a common state."""
import numpy as np
import pytest

from paper_2601_20357_amd import synth

pytestmark = pytest.mark.gpu


def _gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2601_20357_amd import binding
    binding.load()
    return torch, binding


def _to_dev(torch, arr_u16):
    return torch.from_numpy(arr_u16.view(np.int16).copy()).cuda()


def _from_dev(t):
    return t.cpu().numpy().view(np.uint16)


def _close_bf16(got_bits, want_bits, what, layers_before=1):
    """layers_before: how many layers' worth of rounding points lie between the common state and this tensor."""
    got = synth.bf16_to_f32(got_bits).astype(np.float64)
    want = synth.bf16_to_f32(want_bits).astype(np.float64)
    assert np.isfinite(got).all(), what
    row_max = np.abs(want).reshape(want.shape[0], -1).max(axis=1).reshape((-1,) + (1,) * (want.ndim - 1))
    diff = np.abs(got - want)
    assert (diff <= 2.0 ** -6 * row_max + 1e-30).all(), f"{what}: max diff {diff.max()} (row max {row_max.max()})"
    rel_rms = float(np.sqrt((diff ** 2).mean() / max((want ** 2).mean(), 1e-60)))
    assert rel_rms <= 2.0 ** -7, f"{what}: relative RMS difference {rel_rms:.2e}"
    if layers_before <= 2:
        one_step = 2.0 ** -7 * np.maximum(np.abs(want), 2.0 ** -6 * row_max) + 1e-30
        frac = float((diff > one_step).mean())
        assert frac <= 0.01, f"{what}: {frac:.4f} of the entries are more than one bf16 step apart"
    return rel_rms


class BodyPair:
    """The same weights, caches and positions on both sides."""

    def __init__(self, oracle, bc, rows, seed, fill):
        torch, binding = _gpu()
        self.torch, self.binding, self.oracle, self.bc, self.rows = torch, binding, oracle, bc, rows
        self.w = synth.make_body_weights(bc, seed)
        g = np.random.default_rng(900 + seed)
        self.ctx = np.asarray(fill(g), dtype=np.int32)
        assert self.ctx.shape == (rows,)
        shape = (bc.layers, rows, bc.max_ctx, bc.d)
        self.kc = synth.bf16_bits(g.standard_normal(shape, dtype=np.float32))
        self.vc = synth.bf16_bits(g.standard_normal(shape, dtype=np.float32))
        self.cfg = binding.make_body_cfg(layers=bc.layers, d=bc.d, heads=bc.heads, d_ff=bc.d_ff, V=bc.V, max_ctx=bc.max_ctx,
                                         rope_theta=bc.rope_theta, rms_eps=bc.rms_eps)
        self.dev = dict(embed=_to_dev(torch, self.w["embed"]), g_final=torch.from_numpy(self.w["g_final"]).cuda())
        for key in ("wqkv", "wo", "wgu", "wdown"):
            self.dev[key] = [_to_dev(torch, a) for a in self.w[key]]
        for key in ("g_attn", "g_mlp"):
            self.dev[key] = [torch.from_numpy(a).cuda() for a in self.w[key]]
        self.wtab = binding.make_body_weights(self.cfg, self.dev)
        self.ws = torch.empty(binding.tabed_body_workspace_bytes(self.cfg, rows), dtype=torch.uint8, device="cuda")
        binding.tabed_body_workspace_init(self.cfg, rows, self.ws)
        self.d_kc, self.d_vc = _to_dev(torch, self.kc.reshape(-1)), _to_dev(torch, self.vc.reshape(-1))
        self.d_ctx = torch.from_numpy(self.ctx.copy()).cuda()
        self.d_H = torch.zeros(rows * bc.d, dtype=torch.int16, device="cuda")

    def step(self, tokens, token_src=None, token_stride=1, rows_per_token=1):
        """tokens: the token of every row (oracle side); token_src: how the GPU side is told (default: the same list)."""
        torch, bc = self.torch, self.bc
        tokens = np.asarray(tokens, dtype=np.int32)
        before = self.ctx.copy()
        H_o = self.oracle.body_step(layers=bc.layers, d=bc.d, heads=bc.heads, d_ff=bc.d_ff, V=bc.V, max_ctx=bc.max_ctx,
                                    rope_theta=bc.rope_theta, rms_eps=bc.rms_eps, tokens=tokens, ctx_len=self.ctx,
                                    weights=self.w, kcache=self.kc, vcache=self.vc)
        self.ctx = before + 1
        src = torch.from_numpy(tokens).cuda() if token_src is None else token_src
        self.binding.tabed_draft_body_step(self.cfg, self.wtab, self.ws, self.rows, src, token_stride, rows_per_token,
                                           self.d_ctx, self.d_kc, self.d_vc, self.d_H)
        torch.cuda.synchronize()
        assert np.array_equal(self.d_ctx.cpu().numpy(), self.ctx)
        H_g = _from_dev(self.d_H).reshape(self.rows, bc.d)
        changed = _close_bf16(H_g, H_o, "H", bc.layers)
        # the cache rows the step wrote, and nothing else
        kg = _from_dev(self.d_kc).reshape(self.kc.shape)
        vg = _from_dev(self.d_vc).reshape(self.vc.shape)
        r = np.arange(self.rows)
        for name, got, want in (("kcache", kg, self.kc), ("vcache", vg, self.vc)):
            for l in range(bc.layers):
                _close_bf16(got[l, r, before], want[l, r, before], f"{name} layer {l}", l + 1)
            mask = np.ones(want.shape, dtype=bool)
            mask[:, r, before] = False
            assert np.array_equal(got[mask], want[mask]), f"{name}: an entry outside the appended row changed"
        # the next step starts from one state on both sides (the oracle's), so that each step is judged on its own
        self.d_kc.copy_(_to_dev(torch, self.kc.reshape(-1)))
        self.d_vc.copy_(_to_dev(torch, self.vc.reshape(-1)))
        return changed


CASES = [
    # layers, d, heads, d_ff, V, max_ctx, rows
    ("tiny_generic", synth.BodyConfig(layers=2, d=64, heads=4, d_ff=72, V=50, max_ctx=24), 5),
    ("head128", synth.BodyConfig(layers=1, d=256, heads=2, d_ff=512, V=300, max_ctx=40), 33),
    ("d48_three_layers", synth.BodyConfig(layers=3, d=48, heads=3, d_ff=80, V=17, max_ctx=12), 7),
    ("wide_ragged_20_rows", synth.BodyConfig(layers=1, d=256, heads=4, d_ff=1032, V=100, max_ctx=20), 20),
    ("rows_130_many_rows_kernels", synth.BodyConfig(layers=2, d=64, heads=4, d_ff=128, V=90, max_ctx=10), 130),
    ("rows_70_ragged_k", synth.BodyConfig(layers=1, d=72, heads=9, d_ff=200, V=33, max_ctx=8), 70),
    ("d512_skinny", synth.BodyConfig(layers=2, d=512, heads=8, d_ff=1536, V=1000, max_ctx=300), 64),
]


@pytest.mark.parametrize("name,bc,rows", CASES, ids=[c[0] for c in CASES])
def test_body_steps_match_the_oracle(oracle, name, bc, rows):
    pair = BodyPair(oracle, bc, rows, seed=len(name), fill=lambda g: g.integers(0, bc.max_ctx - 3, size=rows))
    pair.ctx[0] = 0                                   # an empty cache: attention over the token itself only
    pair.ctx[-1] = bc.max_ctx - 3                     # the last step fills the cache's last entry
    pair.d_ctx.copy_(pair.torch.from_numpy(pair.ctx))
    g = np.random.default_rng(5)
    for _ in range(3):
        pair.step(g.integers(0, bc.V, size=rows))


def test_body_68m_shape_64_rows(oracle):
    bc = synth.BodyConfig(layers=2, d=768, heads=12, d_ff=3072, V=32000, max_ctx=160)
    rows = 64
    pair = BodyPair(oracle, bc, rows, seed=3, fill=lambda g: g.integers(0, 150, size=rows))
    g = np.random.default_rng(6)
    for _ in range(2):
        pair.step(g.integers(0, bc.V, size=rows))


def test_body_twelve_layers_stay_within_the_rounding_noise_of_the_format(oracle):
    """The depth of the 160M-class draft: the two sides have drifted apart by then, but by no more than bf16's own
    rounding noise (see the module comment)."""
    bc = synth.BodyConfig(layers=12, d=768, heads=12, d_ff=3072, V=2000, max_ctx=40)
    rows = 12
    pair = BodyPair(oracle, bc, rows, seed=8, fill=lambda g: g.integers(0, 36, size=rows))
    rms = pair.step(np.random.default_rng(2).integers(0, bc.V, size=rows))
    assert rms > 0.0                                   # they do differ: the test is not comparing a copy


def test_body_tokens_read_from_the_block_of_drafted_tokens(oracle):
    """Row r = b * n + j is fed draft_tokens[b, i - 1]: a strided view, one token per n rows; out-of-range ids clamp."""
    bc = synth.BodyConfig(layers=1, d=64, heads=4, d_ff=96, V=40, max_ctx=16)
    n, B, gamma, i = 3, 4, 5, 2
    rows = n * B
    pair = BodyPair(oracle, bc, rows, seed=11, fill=lambda g: g.integers(0, 10, size=rows))
    torch = pair.torch
    drafted = np.random.default_rng(1).integers(0, bc.V, size=(B, gamma)).astype(np.int32)
    drafted[1, i - 1] = bc.V + 7                      # clamps to V - 1
    drafted[2, i - 1] = -3                            # clamps to 0
    per_row = np.clip(np.repeat(drafted[:, i - 1], n), 0, bc.V - 1)
    pair.step(per_row, token_src=(torch.from_numpy(drafted.reshape(-1)).cuda(), i - 1), token_stride=gamma, rows_per_token=n)


def test_body_rollback_keeps_the_accepted_prefix():
    torch, binding = _gpu()
    n, B, gamma = 4, 5, 5
    base = torch.arange(100, 100 + n * B, dtype=torch.int32, device="cuda")
    ctx = base + gamma                                # after gamma steps
    k = torch.tensor([0, 2, 4, 5, 3], dtype=torch.int32, device="cuda")
    binding.tabed_draft_body_rollback(n * B, n, gamma, base, k, ctx)
    kept = torch.minimum(k + 1, torch.tensor(gamma, device="cuda")).repeat_interleave(n).to(torch.int32)
    assert torch.equal(ctx, base + kept)


def test_body_rejects_bad_configurations():
    torch, binding = _gpu()
    ok = dict(layers=2, d=64, heads=4, d_ff=72, V=50, max_ctx=24)
    assert binding.tabed_body_workspace_bytes(binding.make_body_cfg(**ok), 8) > 0
    for bad in (dict(layers=0), dict(layers=17), dict(d=60), dict(heads=3), dict(heads=16), dict(d=48, heads=2), dict(d_ff=70), dict(V=0),
                dict(max_ctx=0), dict(max_ctx=8193), dict(rope_theta=0.0), dict(rms_eps=0.0)):
        assert binding.tabed_body_workspace_bytes(binding.make_body_cfg(**{**ok, **bad}), 8) == 0, bad
    assert binding.tabed_body_workspace_bytes(binding.make_body_cfg(**ok), 0) == 0
    assert binding.tabed_body_workspace_bytes(binding.make_body_cfg(**ok), 65536) == 0


def test_rounds_with_the_body_in_the_loop_are_reproducible_bit_for_bit():
    """Body step -> LM head + ensemble + token -> ... -> verify -> rollback, three rounds, run twice from the same
    state: every output identical (the projections' partial sums are added in a fixed order, no atomics), and the
    positions follow the accepted prefix."""
    torch, binding = _gpu()
    bc = synth.BodyConfig(layers=2, d=256, heads=4, d_ff=1024, V=3000, max_ctx=64)
    n, B, gamma = 3, 5, 4
    rows = n * B
    w = synth.make_body_weights(bc, 5)
    dev = dict(embed=_to_dev(torch, w["embed"]), g_final=torch.from_numpy(w["g_final"]).cuda())
    for key in ("wqkv", "wo", "wgu", "wdown"):
        dev[key] = [_to_dev(torch, a) for a in w[key]]
    for key in ("g_attn", "g_mlp"):
        dev[key] = [torch.from_numpy(a).cuda() for a in w[key]]
    bcfg = binding.make_body_cfg(layers=bc.layers, d=bc.d, heads=bc.heads, d_ff=bc.d_ff, V=bc.V, max_ctx=bc.max_ctx)
    cfg = binding.make_cfg(V=bc.V, d=bc.d, n=n, B=B, gamma=gamma, h=4, w_dtype=1, seed=9)
    g = torch.Generator().manual_seed(3)
    Wlm = (torch.randn(bc.V, bc.d, generator=g) * 0.05).to(torch.bfloat16).cuda()
    target = (torch.randn(3, B, gamma + 1, bc.V, generator=g) * 2.0).cuda()
    first_tok = torch.randint(0, bc.V, (3, B), generator=g, dtype=torch.int32).cuda()
    base = torch.randint(0, 20, (rows,), generator=g, dtype=torch.int32).cuda()
    temp = torch.tensor([1.0, 0.0, 0.7, 1.0, 0.0]).cuda()

    def run():
        body = binding.BodyBuffers(bcfg, rows, dev)
        buf = binding.RoundBuffers(cfg)
        body.kcache.copy_(torch.randn(body.kcache.shape, generator=torch.Generator().manual_seed(4)).to(torch.bfloat16))
        body.vcache.copy_(torch.randn(body.vcache.shape, generator=torch.Generator().manual_seed(5)).to(torch.bfloat16))
        body.ctx_base.copy_(base)
        body.ctx_len.copy_(base)
        trace = []
        for rnd in range(3):
            buf.update_weights(rnd == 0, rnd=rnd)
            for pos in range(gamma):
                if pos == 0:
                    binding.tabed_draft_body_step(bcfg, body.table, body.ws, rows, first_tok[rnd], 1, n, body.ctx_len,
                                                  body.kcache, body.vcache, body.H)
                else:
                    binding.tabed_draft_body_step(bcfg, body.table, body.ws, rows, (buf.draft_tokens.view(-1), pos - 1), gamma, n,
                                                  body.ctx_len, body.kcache, body.vcache, body.H)
                buf.draft_step(rnd, pos, Wlm, body.H, temp)
            torch.cuda.synchronize()
            assert torch.equal(body.ctx_len, body.ctx_base + gamma)
            buf.verify(rnd, target[rnd], temp)
            binding.tabed_draft_body_rollback(rows, n, gamma, body.ctx_base, buf.accept_len, body.ctx_len)
            torch.cuda.synchronize()
            kept = torch.clamp(buf.accept_len + 1, max=gamma).repeat_interleave(n)
            assert torch.equal(body.ctx_len, body.ctx_base + kept)
            trace.append([t.clone() for t in (body.H.view(torch.int16), buf.draft_tokens, buf.draft_q, buf.draft_logits,
                                              buf.accept_len, buf.out_tokens, buf.dev, body.ctx_len)])
            body.ctx_base.copy_(body.ctx_len)             # the next round starts where this one stopped
        trace.append([body.kcache.view(torch.int16).clone(), body.vcache.view(torch.int16).clone()])
        return trace

    one, two = run(), run()
    for a, b in zip(one, two):
        for x, y in zip(a, b):
            assert torch.equal(x, y)
    assert all(torch.isfinite(t[2]).all() for t in one[:3])
