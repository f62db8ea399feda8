#!/usr/bin/env python3
"""Benchmark of the TABED hot path on one MI355X.

One step = one speculative-decoding round for all B sequences: tabed_update_weights, gamma x
tabed_draft_step, tabed_verify -- called through the C ABI exactly as a serving loop would.  The workload
is the batched-serving configuration the headline metric is quoted on (V=32000, d=768, n=4, B=16, gamma=5,
h=8, temperature 1); inputs are seeded and synthetic, generated on the GPU before the timed region and
resident in HBM.  The LM-head matrix is rotated over several device copies between rounds so that it is
streamed from HBM the way it would be after the target model's forward pass evicted it.

Prints ONE JSON line: the whole-job rate, the roofline of the dominant kernel (measured with HIP events on
the launch stream in a second, instrumented pass over the same steps) and the CPU oracle timed on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)



def source_digest():
    """Short digest of the kernel sources: a traffic figure measured on other sources is not reported."""
    import hashlib
    h = hashlib.sha256()
    for name in ("device_utils.h", "internal.h", "lmhead.hip", "vocab.hip"):
        with open(os.path.join(ROOT, "paper_2601_20357_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload
    (profiles/<workload>_hbm_traffic.md, FETCH_SIZE and WRITE_SIZE each in a run of its own, scaled by a plain
    device copy).  The summary carries a machine-readable line
        traffic-bytes-per-launch: <kernel>=<bytes> ... sources=<digest>
    Returns (bytes or None, note): None when there is no summary or it was measured on other kernel sources."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.md")
    if not os.path.exists(path):
        return None, "no rocprofv3 --pmc summary for this workload"
    for line in open(path):
        if line.startswith("traffic-bytes-per-launch:"):
            fields = dict(f.split("=", 1) for f in line.split(":", 1)[1].split())
            if fields.get("sources") != source_digest():
                return None, f"{os.path.relpath(path, ROOT)} was measured on other kernel sources ({fields.get('sources')})"
            if kernel in fields:
                return float(fields[kernel]), f"{os.path.relpath(path, ROOT)} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, same kernel sources)"
    return None, "summary holds no figure for this kernel"


HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="serving", choices=["tiny", "llava", "serving", "lvlm", "stress"])
    ap.add_argument("--pool", type=int, default=8, help="distinct pre-generated rounds (and W copies) cycled through")
    ap.add_argument("--w-copies", type=int, default=8, help="device copies of W rotated per round (1 = warm cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rounds", type=int, default=0,
                    help="rounds of the oracle's timed sample (0 = a workload-dependent default of 10-30 s)")
    ap.add_argument("--print-source-digest", action="store_true", help="print the kernel-source digest and exit")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--separate-update", action="store_true",
                    help="call tabed_update_weights at the start of every round instead of letting tabed_verify "
                         "open the next round (window push + next weights) in its last workgroup")
    ap.add_argument("--launch", default="graph", choices=["graph", "eager"],
                    help="graph: the pool's rounds are captured once into a HIP graph (stream capture of the same "
                         "C-ABI calls) and replayed; eager: every call is issued from Python each round")
    ap.add_argument("--tree-width", type=int, default=1,
                    help="token tree of this width (2 or 3) instead of the chain: every draft step also draws the "
                         "siblings, tabed_verify_tree verifies; the window update is then a call of its own")
    ap.add_argument("--draft-body", default="none", choices=["none", "68m", "160m"],
                    help="run the draft model's body (random weights) in front of every LM-head call instead of "
                         "feeding pre-generated hidden states; reports rounds/s of body + head + verify")
    ap.add_argument("--policy", type=int, default=0, help="weight policy (0 softmax of 1/e, 1 static, 2 two-draft grid, 3 random)")
    ap.add_argument("--distance", type=int, default=0, help="0 KL, 1 total variation")
    ap.add_argument("--drafts", type=int, default=0, help="override the workload's number of drafts n (2 for --policy 2)")
    ap.add_argument("--hidden", type=int, default=0, help="override the workload's draft hidden size d")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MB",
                    help="only run a plain device copy of MB megabytes 10 times: the known-size kernel against "
                         "which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    return ap.parse_args()


def gen_inputs(wl, pool, w_copies, device):
    """Same recipe as paper_2601_20357_amd.synth, drawn with torch on the GPU (inputs, not the method)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(1000 * wl.cfg_id)
    sd = torch.float32 if wl.w_dtype == 0 else torch.bfloat16
    W = (torch.randn((wl.V, wl.d), generator=g, device=device) * 0.02).to(sd)
    Ws = [W] + [W.clone() for _ in range(w_copies - 1)]
    if wl.temperature == "mixed07":
        temp = torch.zeros(wl.B, device=device); temp[1::2] = 0.7
    elif wl.temperature == "greedy":
        temp = torch.zeros(wl.B, device=device)
    else:
        temp = torch.ones(wl.B, device=device)
    sig = torch.rand(wl.B, generator=g, device=device) * 1.3 + 0.2
    Hs, Ts = [], []
    for r in range(pool):
        H = torch.randn((wl.gamma + 1, wl.B, wl.n, wl.d), generator=g, device=device).to(sd)
        shape = (wl.B, wl.gamma + 1, wl.V)
        if wl.target == "independent":
            tgt = torch.randn(shape, generator=g, device=device) * wl.sigma
        else:
            jstar = (r // wl.switch_every) % wl.n if wl.target == "switching" else 0
            base = torch.einsum("ibk,vk->biv", H[:, :, jstar, :].float(), W.float())
            if wl.target == "student_t":
                z = torch.randn(shape, generator=g, device=device)
                chi = torch.randn((3,) + shape, generator=g, device=device).pow(2).sum(0)
                noise = z / (chi / 3).sqrt() * wl.sigma
            elif wl.target == "per_seq_sigma":
                noise = torch.randn(shape, generator=g, device=device) * sig[:, None, None]
            else:
                noise = torch.randn(shape, generator=g, device=device) * wl.sigma
            tgt = base + noise
        Hs.append(H.contiguous())
        Ts.append(tgt.float().contiguous())
    return Ws, Hs, Ts, temp.float().contiguous()


def gen_leaf_logits(wl, Ws, Hs, width, device):
    """Target logits after the leaves of a token tree, [B,gamma,width-1,V] per pooled round: the recipe of the next
    position's target row with a noise draw of its own (see synth.make_tree_leaves)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(1000 * wl.cfg_id + 7)
    out = []
    for r, H in enumerate(Hs):
        jstar = (r // wl.switch_every) % wl.n if wl.target == "switching" else 0
        base = torch.einsum("ibk,vk->biv", H[1:, :, jstar, :].float(), Ws[0].float())      # [B,gamma,V]
        noise = torch.randn((wl.B, wl.gamma, width - 1, wl.V), generator=g, device=device) * (wl.sigma or 0.8)
        out.append((base[:, :, None, :] + noise).float().contiguous())
    return out


CPU_SAMPLE = {"tiny": (2000, None), "llava": (120, None), "serving": (60, None), "lvlm": (4, None), "stress": (1, 8)}


def cpu_baseline(wl, rounds):
    """The oracle as it stands, on this machine's host cores, on a bounded sample of the same workload: `rounds` full
    rounds, or -- where one round of all sequences takes minutes (stress) -- the first few sequences of a round,
    scaled by their share (the oracle's work is per sequence)."""
    import numpy as np
    import oracle
    from paper_2601_20357_amd import synth
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import harness
    default_rounds, seqs = CPU_SAMPLE[wl.name]
    rounds = rounds or default_rounds
    W = synth.make_lm_head(wl)
    temp = synth.make_temperature(wl)
    inputs = [synth.make_round(wl, W, r) for r in range(rounds)]
    wl_o = wl
    if seqs is not None and seqs < wl.B:
        wl_o = synth.scaled(wl, B=seqs)
        temp = temp[:seqs]
        inputs = [(np.ascontiguousarray(H[:, :seqs]), np.ascontiguousarray(t[:seqs])) for H, t in inputs]
    side = harness.OracleSide(oracle, wl_o)
    t0 = time.perf_counter()
    for r, (H, tgt) in enumerate(inputs):
        side.round(r, W, H, tgt, temp)
    dt = time.perf_counter() - t0
    share = wl_o.B / wl.B
    what = (f"{rounds} full rounds of the {wl.name} workload (all B={wl.B} sequences)" if share == 1.0 else
            f"{rounds} round(s) of the first {wl_o.B} of the {wl.name} workload's {wl.B} sequences, rate scaled by {share:.4f}")
    # the same oracle on ONE thread, on a few of the same rounds
    cores = oracle.threads()
    few = max(2, rounds // 15)
    oracle.set_threads(1)
    side1 = harness.OracleSide(oracle, wl_o)
    t1 = time.perf_counter()
    for r, (H, tgt) in enumerate(inputs[:few]):
        side1.round(r, W, H, tgt, temp)
    dt1 = time.perf_counter() - t1
    oracle.set_threads(cores)
    return {"value": rounds / dt * share, "unit": "steps/s", "cores": cores, "kind": "oracle",
            "sample": f"{what}, {dt:.1f} s",
            "one_thread": {"value": few / dt1 * share, "unit": "steps/s", "sample": f"the first {few} of those rounds, {dt1:.1f} s"}}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.print_source_digest:
        print(source_digest())
        return
    import torch
    from paper_2601_20357_amd import binding, synth

    if args.calibrate_copy:
        nbytes = args.calibrate_copy << 20
        src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "device copy", "bytes_read_per_launch": nbytes,
                          "bytes_written_per_launch": nbytes, "launches": 10}), flush=True)
        return

    wl = synth.WORKLOADS[args.workload]
    if args.drafts:
        wl = synth.scaled(wl, n=args.drafts)
    if args.hidden:
        wl = synth.scaled(wl, d=args.hidden)
    device = "cuda:0"
    torch.cuda.set_device(0)
    binding.load()
    Ws, Hs, Ts, temp = gen_inputs(wl, args.pool, args.w_copies, device)
    cfg = binding.make_cfg(V=wl.V, d=wl.d, n=wl.n, B=wl.B, gamma=wl.gamma, h=wl.h, w_dtype=wl.w_dtype, seed=0,
                           policy=args.policy, distance=args.distance)
    buf = binding.RoundBuffers(cfg, device)

    tree = args.tree_width > 1
    if tree:
        args.separate_update = True
        buf.enable_tree(args.tree_width)
        Ls = gen_leaf_logits(wl, Ws, Hs, args.tree_width, device)
    upd_first = buf.prepare_update_weights(True)
    upd = buf.prepare_update_weights(False)
    body = None
    if args.draft_body != "none":
        if tree or wl.w_dtype != 1:
            sys.exit("bench.py: --draft-body needs a bf16 workload and --tree-width 1")
        import numpy as np
        bc = synth.scaled_body(synth.BODIES[args.draft_body], d=wl.d, V=wl.V)
        bw = synth.make_body_weights(bc, 0)
        as_dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(device)
        tensors = {k: ([as_dev(a) for a in v] if isinstance(v, list) else as_dev(v)) for k, v in bw.items()}
        bcfg = binding.make_body_cfg(layers=bc.layers, d=bc.d, heads=bc.heads, d_ff=bc.d_ff, V=bc.V, max_ctx=bc.max_ctx,
                                     rope_theta=bc.rope_theta, rms_eps=bc.rms_eps)
        body = binding.BodyBuffers(bcfg, wl.n * wl.B, tensors, device)
        g = torch.Generator(device="cpu").manual_seed(11)
        # contexts of a few hundred tokens (prompt, image or caption tokens, what was generated so far), different
        # for every drafting method of a sequence; the caches hold unit-variance keys and values up to there
        body.ctx_base.copy_(torch.randint(256, 768, (wl.n * wl.B,), generator=g, dtype=torch.int32))
        body.ctx_len.copy_(body.ctx_base)
        body.kcache.normal_()
        body.vcache.normal_()
        first_tokens = torch.randint(0, wl.V, (args.pool, wl.B), generator=g, dtype=torch.int32).to(device)
    def make_slots(per_step_rotation):
        out = []
        for r in range(args.pool):
            drafts = []
            for pos in range(wl.gamma):
                # default: one W copy per round (a round's gamma calls find W where the previous call left it,
                # as they would with a 68M-class draft body between them); per-step: every call a fresh copy
                W = Ws[(r * wl.gamma + pos) % len(Ws)] if per_step_rotation else Ws[r % len(Ws)]
                if body is not None:
                    # position 0 is fed the round's first token, position i > 0 the token drafted at i - 1
                    drafts.append(body.prepare_step(first_tokens[r], 0, 1, wl.n) if pos == 0 else
                                  body.prepare_step(buf.draft_tokens, pos - 1, wl.gamma, wl.n))
                drafts.append(buf.prepare_draft_step(0, pos, W, body.H if body is not None else Hs[r][pos], temp))
                if tree:
                    drafts.append(buf.prepare_draft_siblings(0, pos, temp))
            ver = (buf.prepare_verify_tree(0, Ts[r], Ls[r], temp) if tree else
                   buf.prepare_verify(0, Ts[r], temp, fused_update=not args.separate_update))
            out.append((drafts, ver))
        return out

    # after verification the caches keep the accepted prefix.  ctx_base stays what it was at the start of the run
    # (a serving loop would move it on by the tokens emitted), so that every round works at the recipe's context length
    rollback = body.prepare_rollback(wl.n, wl.gamma, buf.accept_len) if body is not None else None

    slots = make_slots(False)

    state = {"step": 0}

    def step():
        s = state["step"]
        drafts, ver = slots[s % args.pool]
        if s == 0:
            upd_first()                       # opens the first round: empty window, equal weights
        elif args.separate_update:
            upd.set_round(s)
            upd()
        for c in drafts:
            c.set_round(s)
            c()
        ver.set_round(s)
        ver()
        if rollback is not None:
            rollback()
        state["step"] = s + 1

    def timed(k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            step()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    launch = args.launch
    every = [upd, upd_first] + [c for drafts, ver in slots for c in drafts + [ver]] + ([rollback] if rollback else [])

    def set_stream(handle):
        import ctypes as C
        for c in every:
            c.args[-1] = C.c_void_p(handle)

    if launch == "graph":
        try:
            # Capture one pass over the pool (pool x (1 + gamma) C-ABI calls) on a side stream and replay it: the
            # library enqueues only kernels (no memset, no allocation, no sync), so the same calls are capturable
            # as they are.  K steps = K // pool replays of that graph plus one replay of a second graph holding
            # the first K % pool rounds of the pool.  The round counter of a captured call is fixed, so the Philox
            # uniforms repeat with the pool, like the inputs do; the window state still evolves across replays.
            side = torch.cuda.Stream()
            set_stream(side.cuda_stream)
            # (a short run, K <= 128, is one graph of its own: a single launch for all K steps)
            unit = args.steps if args.steps <= 128 else args.pool
            full, rem = args.steps // unit, args.steps % unit
            graph, graph_rem = torch.cuda.CUDAGraph(), (torch.cuda.CUDAGraph() if rem else None)
            with torch.cuda.stream(side):
                state["step"] = args.pool * ((state["step"] + args.pool - 1) // args.pool)   # a replay starts at slot 0
                for _ in range(args.pool):
                    step()                        # once eagerly on the side stream
                side.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    for _ in range(unit):
                        step()
                if rem:
                    with torch.cuda.graph(graph_rem, stream=side):
                        for _ in range(rem):
                            step()
                    state["step"] += unit - rem
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(full):
                graph.replay()
            if rem:
                graph_rem.replay()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            set_stream(torch.cuda.current_stream().cuda_stream)   # back to the default stream for the instrumented pass
        except Exception as exc:                   # a capture that fails must not cost the measurement
            set_stream(torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            launch = f"eager (graph capture failed: {type(exc).__name__})"
            dt = timed(args.steps)
    else:
        dt = timed(args.steps)
    ms_per_step = dt / args.steps * 1e3
    # tokens emitted per round and sequence, averaged over one more (untimed) pass over the pool
    emitted_sum = 0.0
    for _ in range(args.pool):
        step()
        torch.cuda.synchronize()
        emitted_sum += float(buf.n_out.float().mean().item()) if tree else float(buf.accept_len.float().mean().item()) + 1.0
    emitted = emitted_sum / args.pool

    # ---- second, instrumented pass over the same steps: per-kernel HIP-event timing on the launch stream
    kernels = {}
    roofline = None
    M = wl.n * wl.B
    esz = 4 if wl.w_dtype == 0 else 2
    NT = (wl.V + 31) // 32
    n_sampling = int((temp > 0).sum().item())
    # algorithmic bytes per launch: what the method must move, each logit written once and read once
    alg_bytes = {
        "lmhead": wl.V * wl.d * esz + M * wl.V * 4 + M * wl.d * esz,            # W once + logits once + H
        "sample": M * NT * 8 + n_sampling * wl.n * 32 * 4                         # softmax partials + one tile per row
                  + (wl.B - n_sampling) * wl.n * wl.V * 4,                        # greedy rows: the whole row
        "stats": wl.B * (wl.gamma + 1) * wl.V * 4 + wl.gamma * M * wl.V * 4,     # target rows + draft rows
        "resid": n_sampling * (1 + wl.n) * wl.V * 4,                              # one target row + n draft rows
        "dist": wl.B * wl.gamma * (1 + wl.n) * wl.V * 4,
    }
    body_weight_bytes = 0
    if body is not None:                       # what a body step must stream: every layer's matrices once
        body_weight_bytes = bc.layers * 2 * (3 * bc.d * bc.d + bc.d * bc.d + 3 * bc.d * bc.d_ff)
    lm_bytes = alg_bytes["lmhead"]
    lm_flops = 2.0 * M * wl.d * wl.V
    if not args.no_kernel_timing:
        binding.tabed_prof_reset()
        binding.tabed_prof_enable(True)
        dt_inst = timed(args.steps)
        for _ in range(200):                       # an empty kernel timed the same way: the floor of the method
            binding.tabed_prof_null()
        binding.tabed_prof_enable(False)
        for kid in range(binding.K_COUNT):
            ms, cnt = binding.tabed_prof_read(kid)
            if cnt:
                name = binding.tabed_kernel_name(kid)
                us = ms / cnt * 1e3
                kernels[name] = {"avg_us": us, "launches": cnt}
                if name == "body":                 # all kernels of one tabed_draft_body_step together
                    kernels[name].update(launches_per_step=cnt / (args.steps * wl.gamma),
                                         per_step_us=ms * 1e3 / (args.steps * wl.gamma),
                                         weight_bytes_per_step=body_weight_bytes,
                                         weights_gbs=body_weight_bytes / (ms * 1e-3 / (args.steps * wl.gamma)) / 1e9)
                if name in alg_bytes:
                    gbs = alg_bytes[name] / (us * 1e-6) / 1e9
                    kernels[name].update(algorithmic_bytes=alg_bytes[name], achieved_gbs=gbs,
                                         frac_of_hbm_peak=gbs / HBM_PEAK_GBS)
        # the same pass with a fresh W copy for EVERY LM-head launch: all launches stream W from HBM
        saved = list(slots)
        slots[:] = make_slots(True)
        binding.tabed_prof_reset()
        binding.tabed_prof_enable(True)
        timed(min(args.steps, 96))
        binding.tabed_prof_enable(False)
        cold_ms, cold_cnt = binding.tabed_prof_read(binding.K_LMHEAD)
        cold_us = cold_ms / max(cold_cnt, 1) * 1e3
        slots[:] = saved
        lm_us = kernels["lmhead"]["avg_us"]                 # events attached to the dispatch: the kernel's own time
        null_us = kernels.get("null", {}).get("avg_us", 0.0)
        gbs = lm_bytes / (lm_us * 1e-6) / 1e9
        tflops = lm_flops / (lm_us * 1e-6) / 1e12
        kernels["lmhead"].update(flops=lm_flops, achieved_tflops=tflops, frac_of_bf16_mfma_peak=tflops / MFMA_BF16_PEAK_TFLOPS)
        # the LM head is the dominant kernel; it is bound by the matrix cores only when its intensity
        # (flop per algorithmic byte) exceeds the ridge of the chip, i.e. at several hundred rows
        mfma_bound = wl.w_dtype == 1 and lm_flops / lm_bytes > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
        traffic, traffic_note = measured_traffic(wl.name, "lmhead")
        roofline = {"kernel": "lmhead"}
        if mfma_bound:
            roofline.update(bound="mfma", achieved=tflops, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                            frac=tflops / MFMA_BF16_PEAK_TFLOPS)
        else:
            roofline.update(bound="hbm", achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS)
        roofline.update(traffic=traffic, traffic_source=traffic_note,
                        algorithmic_bytes_per_launch=lm_bytes, flops_per_launch=lm_flops, avg_launch_us=lm_us,
                        empty_kernel_us=null_us,
                        every_launch_fresh_w={"avg_launch_us": cold_us, "achieved_gbs": lm_bytes / (cold_us * 1e-6) / 1e9,
                                              "frac_of_hbm_peak": lm_bytes / (cold_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
                        hbm_gbs=gbs, frac_of_hbm_peak=gbs / HBM_PEAK_GBS,
                        mfma_tflops=tflops, mfma_frac_of_bf16_peak=tflops / MFMA_BF16_PEAK_TFLOPS,
                        instrumented_ms_per_step=dt_inst / args.steps * 1e3)

    round_bytes = wl.gamma * (lm_bytes + alg_bytes["sample"]) + alg_bytes["stats"] + alg_bytes["resid"] \
        + (alg_bytes["dist"] if (args.distance != 0 or args.policy == 2) else 0)
    out = {
        "metric": ("ensemble-draft+verify steps/sec at V=32k,n=4,B=16; HBM GB/s & MFMA % of peak"
                   if wl.name == "serving" and not tree and body is None else "ensemble-draft+verify steps/sec"),
        "value": args.steps / dt, "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.w_dtype == 1 else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: V={wl.V} d={wl.d} n={wl.n} B={wl.B} gamma={wl.gamma} h={wl.h} "
                               f"temperature={wl.temperature} policy={args.policy} distance={args.distance}",
                   "pool_rounds": args.pool, "w_copies": args.w_copies,
                   "calls_per_step": (2 if args.separate_update else 1) + wl.gamma * (2 if tree or body is not None else 1)
                                     + (1 if body is not None else 0), "launch": launch,
                   "window_update": "separate call" if args.separate_update else "fused into tabed_verify",
                   "tree_width": args.tree_width, "draft_body": args.draft_body},
        "roofline": roofline,
        "cpu_baseline": None,
        "detail": {"kernels": kernels, "mean_tokens_per_round": emitted,
                   "round_algorithmic_bytes": round_bytes,
                   "round_frac_of_hbm_roofline": round_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "kernel_source_digest": source_digest()},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_rounds)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
