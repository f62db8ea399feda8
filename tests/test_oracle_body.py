"""Pin of the draft-body oracle: the same decode steps built from library operators in fp64 (embedding, linear,
rms_norm, scaled_dot_product_attention, silu; the rotary embedding as a complex multiplication), with the same
bf16 / fp32 storage points.  Another author's operators, another formulation of the rotation and of attention:
a wrong pairing of rotary dimensions, a transposed projection, a missing 1/sqrt(head_dim), a cache row written at
the wrong position or a swapped gate / up half would all show."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2601_20357_amd import synth


def _bf(x_bits):
    return torch.from_numpy(synth.bf16_to_f32(np.asarray(x_bits)).astype(np.float64))


def _store_bf16(x):
    return x.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def _store_f32(x):
    return x.to(torch.float32).to(torch.float64)


def _reference_step(bc, w, tokens, ctx_len, kc, vc):
    """kc, vc: float64 tensors [layers, M, max_ctx, d] holding bf16-representable values; updated in place."""
    M, hd = len(tokens), bc.d // bc.heads
    x = F.embedding(torch.as_tensor(tokens, dtype=torch.long), _bf(w["embed"]))
    pos = torch.as_tensor(ctx_len, dtype=torch.float64)
    inv_freq = bc.rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(M, hd // 2, dtype=torch.float64), pos[:, None] * inv_freq[None, :])     # e^{i pos w}
    for l in range(bc.layers):
        h = _store_bf16(F.rms_norm(x, (bc.d,), torch.from_numpy(w["g_attn"][l].astype(np.float64)), bc.rms_eps))
        qkv = _store_f32(F.linear(h, _bf(w["wqkv"][l])))
        q, k, v = [t.reshape(M, bc.heads, hd) for t in qkv.split(bc.d, dim=1)]
        cplx = lambda t: torch.complex(t[..., : hd // 2], t[..., hd // 2:])
        uncplx = lambda z: torch.cat([z.real, z.imag], dim=-1)
        q = _store_f32(uncplx(cplx(q) * rot[:, None, :]))
        k = _store_bf16(uncplx(cplx(k) * rot[:, None, :]))
        v = _store_bf16(v)
        out = torch.zeros(M, bc.d, dtype=torch.float64)
        for r in range(M):
            p = int(ctx_len[r])
            kc[l, r, p] = k[r].reshape(-1)
            vc[l, r, p] = v[r].reshape(-1)
            K = kc[l, r, : p + 1].reshape(p + 1, bc.heads, hd).transpose(0, 1)      # [heads, p+1, hd]
            Vv = vc[l, r, : p + 1].reshape(p + 1, bc.heads, hd).transpose(0, 1)
            o = F.scaled_dot_product_attention(q[r][:, None, :], K, Vv)             # [heads, 1, hd]
            out[r] = o.reshape(-1)
        x = _store_f32(x + _store_f32(F.linear(_store_bf16(out), _bf(w["wo"][l]))))
        h2 = _store_bf16(F.rms_norm(x, (bc.d,), torch.from_numpy(w["g_mlp"][l].astype(np.float64)), bc.rms_eps))
        gu = _store_f32(F.linear(h2, _bf(w["wgu"][l])))
        act = _store_bf16(F.silu(gu[:, : bc.d_ff]) * gu[:, bc.d_ff:])
        x = _store_f32(x + _store_f32(F.linear(act, _bf(w["wdown"][l]))))
    return _store_bf16(F.rms_norm(x, (bc.d,), torch.from_numpy(w["g_final"].astype(np.float64)), bc.rms_eps))


@pytest.mark.parametrize("shape", [(2, 64, 4, 96, 50, 24), (1, 128, 2, 160, 31, 40), (3, 48, 3, 80, 17, 12)],
                         ids=["2x64", "1x128", "3x48"])
def test_body_step_matches_library_operators(oracle, shape):
    layers, d, heads, d_ff, V, max_ctx = shape
    bc = synth.BodyConfig(layers=layers, d=d, heads=heads, d_ff=d_ff, V=V, max_ctx=max_ctx)
    w = synth.make_body_weights(bc, seed=d)
    rng = np.random.default_rng(d)
    M = 5
    ctx = rng.integers(0, max_ctx - 4, M).astype(np.int32)
    kc = synth.bf16_bits(rng.standard_normal((layers, M, max_ctx, d)).astype(np.float32))
    vc = synth.bf16_bits(rng.standard_normal((layers, M, max_ctx, d)).astype(np.float32))
    kc_ref, vc_ref = _bf(kc).clone(), _bf(vc).clone()
    for step in range(3):                                   # three tokens in a row: the cache rows just written are read back
        tokens = rng.integers(0, V, M).astype(np.int32)
        H = oracle.body_step(layers=layers, d=d, heads=heads, d_ff=d_ff, V=V, max_ctx=max_ctx, rope_theta=bc.rope_theta,
                             rms_eps=bc.rms_eps, tokens=tokens, ctx_len=ctx, weights=w, kcache=kc, vcache=vc)
        H_ref = _reference_step(bc, w, tokens, ctx, kc_ref, vc_ref)
        got = _bf(H)
        # both sides are fp64 with identical storage points: equal up to the rare bf16 rounding flipped by
        # a different summation order
        diff = (got - H_ref).abs()
        assert float((diff > 0).double().mean()) < 0.02, float((diff > 0).double().mean())
        assert float(diff.max()) <= 2.0 ** -7 * float(H_ref.abs().max())
        for a, b in ((kc, kc_ref), (vc, vc_ref)):
            dd = (_bf(a) - b).abs()
            assert float((dd > 0).double().mean()) < 0.002 and float(dd.max()) <= 2.0 ** -7 * float(b.abs().max())
        # only the row at position ctx of every (layer, row) changed
        ctx = ctx + 1
