"""tabed_draft_step_static (the draft step on the library's built-in scratch buffer, for callers that cannot
allocate) against tabed_draft_step with a caller-provided workspace: same kernels, so every output must be
bit-identical -- on two calls in a row, the second with a smaller input, because the built-in buffer keeps the
previous call's contents."""
import numpy as np
import pytest
import torch

from paper_2601_20357_amd import binding, synth

import harness
from harness import DEV

pytestmark = pytest.mark.gpu


def _one_position(wl, seed, pos, rnd):
    """Both entry points on the same inputs; returns the two sets of outputs."""
    cfg = harness.cfg_of(wl, seed=seed)
    assert binding.tabed_workspace_bytes(cfg) <= binding.STATIC_SCRATCH_BYTES
    W = synth.make_lm_head(wl)
    H, _ = synth.make_round(wl, W, rnd)
    W_t, H_t = harness.to_dev_store(W, wl.w_dtype), harness.to_dev_store(H[pos], wl.w_dtype)
    temp = torch.from_numpy(synth.make_temperature(wl, "mixed07")).to(DEV)
    g = torch.Generator(device="cpu").manual_seed(seed)
    w = torch.rand((wl.B, wl.n), generator=g)
    weights = (w / w.sum(1, keepdim=True)).float().to(DEV)
    outs = []
    for static in (False, True):
        buf = binding.RoundBuffers(cfg, DEV)
        buf.weights.copy_(weights)
        for t in (buf.draft_logits, buf.draft_q):
            t.fill_(float("nan"))
        buf.draft_tokens.fill_(-5)
        if static:
            binding.tabed_draft_step_static(cfg, rnd, pos, W_t, H_t, buf.weights, temp, buf.draft_logits, buf.draft_lse,
                                            buf.draft_tokens, buf.draft_q, buf.draft_flags)
        else:
            binding.tabed_draft_step(cfg, buf.ws, rnd, pos, W_t, H_t, buf.weights, temp, buf.draft_logits, buf.draft_lse,
                                     buf.draft_tokens, buf.draft_q, buf.draft_flags)
        torch.cuda.synchronize()
        outs.append(dict(logits=buf.draft_logits[pos].clone(), lse=buf.draft_lse[pos].clone(),
                         tokens=buf.draft_tokens[:, pos].clone(), q=buf.draft_q[:, pos].clone(),
                         flags=buf.draft_flags[:, pos].clone()))
    return outs


def test_static_scratch_entry_point_matches_workspace_entry_point_twice():
    big = synth.scaled(synth.WORKLOADS["serving"], gamma=2, cfg_id=301)              # V=32000, d=768, n=4, B=16
    small = synth.scaled(synth.WORKLOADS["serving"], V=5003, d=512, n=3, B=5, gamma=2, cfg_id=302)
    for wl, seed, pos, rnd in ((big, 1, 1, 7), (small, 2, 0, 8)):
        print(f"static scratch: V={wl.V} d={wl.d} n={wl.n} B={wl.B} pos={pos}", flush=True)
        ref, got = _one_position(wl, seed, pos, rnd)
        for key in ref:
            assert torch.equal(ref[key], got[key]), (wl.V, key)
        assert int((ref["tokens"] >= 0).all()) and torch.isfinite(ref["logits"]).all()


def test_static_scratch_rejects_a_configuration_that_does_not_fit():
    wl = synth.WORKLOADS["stress"]
    cfg = harness.cfg_of(wl)
    assert binding.tabed_workspace_bytes(cfg) > binding.STATIC_SCRATCH_BYTES
    one = torch.zeros(16, device=DEV)
    with pytest.raises(binding.TabedError, match="built-in buffer"):
        # the size check comes before any pointer is used: small placeholders are never dereferenced
        binding.load().tabed_draft_step_static.argtypes  # noqa: B018 (keeps the symbol lookup explicit)
        rc = binding.load().tabed_draft_step_static(
            __import__("ctypes").byref(cfg), 0, 0, *([one.data_ptr()] * 10), None)
        binding._check(rc, "tabed_draft_step_static")
