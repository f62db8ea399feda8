"""Do the CPU pins have teeth?  Plant one mistake at a time in a COPY of the oracle's C file (the kind of slip a
re-implementation makes: a sign, a direction, a transposed operand, an off-by-one), build the copy, and run the
pin tests against it in a child process: every mutant must make at least one pin fail.  Everything here runs on
the CPU and touches only oracle/."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "tabed_oracle.c")
SRC_BODY = os.path.join(ROOT, "oracle", "tabed_body_oracle.c")
PIN_FILES = ["tests/test_oracle_blocks.py", "tests/test_oracle_sd.py", "tests/test_oracle_tree.py"]
BODY_PIN_FILES = ["tests/test_oracle_body.py"]

# (name, text in the oracle, replacement, replace every occurrence?)
MUTANTS = [
    ("temperature multiplies instead of divides", "/ T_eff", "* T_eff", True),
    ("residual sign", "f[v] = fmax(0.0, p[v] - f[v]);", "f[v] = fmax(0.0, f[v] - p[v]);", False),
    ("accept direction", "ok = lhs < py;", "ok = lhs > py;", False),
    ("ensemble in logit space",
     "for (int j = 0; j < n; ++j) acc += (double)w[j] * q[(size_t)j * V + v];\n        q_ens[v] = acc;",
     "for (int j = 0; j < n; ++j) acc += (double)w[j] * log(q[(size_t)j * V + v]);\n        q_ens[v] = exp(acc);", False),
    ("KL direction", "acc += p[v] * (logp[v] - logq[v]);", "acc += exp(logq[v]) * (logq[v] - logp[v]);", False),
    ("transposed W", "wrow[k] = load_elem(W, w_dtype, (size_t)v * d + k);",
     "wrow[k] = load_elem(W, w_dtype, (size_t)k * V + v);", False),
    ("weights use e instead of 1/e", "x[j] = (1.0 / fmax(e, eps)) / tau_w;", "x[j] = (fmax(e, eps)) / tau_w;", False),
    ("window off by one", "if (ring_count[b] < h) ring_count[b]++;", "if (ring_count[b] < h - 1) ring_count[b]++;", False),
    ("positions after the rejection enter the window", "n_valid[b] = k + 1 < gamma ? k + 1 : gamma;",
     "n_valid[b] = gamma;", False),
    ("bonus token from the wrong row", "oracle_softmax(Lt + (size_t)gamma * V, V, T_eff, p, NULL);",
     "oracle_softmax(Lt + (size_t)(gamma - 1) * V, V, T_eff, p, NULL);", False),
    ("CDF crossing uses >=", "if (c > target) {", "if (c >= target) {", False),
    ("arg-max takes the highest index on ties", "for (int v = 1; v < V; ++v) if (f[v] > f[best]) best = v;",
     "for (int v = 1; v < V; ++v) if (f[v] >= f[best]) best = v;", False),
    ("total variation without the half", "return 0.5 * acc;", "return acc;", False),
    ("grid candidate weights swapped", "f[v] = w0 * q[v] + w1 * q[(size_t)V + v];",
     "f[v] = w1 * q[v] + w0 * q[(size_t)V + v];", False),
    ("grid arg-max instead of arg-min", "if (e < ebest) { ebest = e; best = c; }",
     "if (e > ebest || c == 0) { ebest = e; best = c; }", False),
    ("Philox key schedule swapped", "k0 += W0; k1 += W1;", "k0 += W1; k1 += W0;", False),
    ("Philox multipliers swapped", "uint64_t p0 = (uint64_t)M0 * c0;\n        uint64_t p1 = (uint64_t)M1 * c2;",
     "uint64_t p0 = (uint64_t)M1 * c0;\n        uint64_t p1 = (uint64_t)M0 * c2;", False),
    ("Philox output words rotated", "out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;",
     "out[0] = c1; out[1] = c2; out[2] = c3; out[3] = c0;", False),
    ("23-bit uniforms", "(float)(out[word & 3] >> 8) * (1.0f / 16777216.0f)",
     "(float)(out[word & 3] >> 9) * (1.0f / 8388608.0f)", False),
    ("tree: residual level without the renormalisation", "f[v] = fmax(0.0, f[v] / Zprev - q_ens[v]); Z += f[v];",
     "f[v] = fmax(0.0, f[v] - q_ens[v]); Z += f[v];", False),
    ("tree: sibling test without the level's mass", "double lhs = (double)u * qy * Z;", "double lhs = (double)u * qy;", False),
    ("tree: the last sibling is never tried", "if (c > S) break;                            /* every candidate rejected: f = f_width */",
     "if (c >= S) break;", False),
    ("tree: last level skipped", "for (int c = 1; c <= width; ++c) {", "for (int c = 1; c <= S; ++c) {", False),
    ("tree: bonus after a leaf from the trunk's next row",
     "oracle_softmax(leaf_logits + (((size_t)b * gamma + k) * S + (accepted - 1)) * V, V, T_eff, p, NULL);",
     "oracle_softmax(target_logits + ((size_t)b * (gamma + 1) + k + 1) * V, V, T_eff, p, NULL);", False),
    ("tree: siblings reuse the trunk's uniform",
     "(uint32_t)pos + (uint32_t)s * ORACLE_SIB_STRIDE, 0);", "(uint32_t)pos, 0);", False),
    ("tree: greedy siblings may repeat the trunk", "if (trunk >= 0 && trunk < V) rest[trunk] = -1.0;", "", False),
    ("Eq. 1 without the +1", "return block_eff / (gamma * tq_over_tp + 1.0);", "return block_eff / (gamma * tq_over_tp);", False),
]


# mistakes planted in the draft-body oracle (tabed_body_oracle.c), caught by its library-operator pin
BODY_MUTANTS = [
    ("body: rotary pairs (i, i+1) instead of (i, i + head_dim/2)", "double q0 = q[i], q1 = q[i + hd / 2], k0 = k[i], k1 = k[i + hd / 2];",
     "double q0 = q[i], q1 = q[(i + 1) % hd], k0 = k[i], k1 = k[i + hd / 2];", False),
    ("body: scores not scaled by 1/sqrt(head_dim)", "sc[t] = acc / sqrt((double)hd);", "sc[t] = acc;", False),
    ("body: gate and up halves swapped", "act[f] = round_bf16(gu[f] / (1.0 + exp(-gu[f])) * gu[d_ff + f]);",
     "act[f] = round_bf16(gu[d_ff + f] / (1.0 + exp(-gu[d_ff + f])) * gu[f]);", False),
    ("body: the new key is not part of its own attention", "for (int t = 0; t <= pos; ++t) { sc[t] = exp(sc[t] - mx); Z += sc[t]; }",
     "sc[pos] = -INFINITY; for (int t = 0; t <= pos; ++t) { sc[t] = exp(sc[t] - mx); Z += sc[t]; }", False),
    ("body: rotation angle with the wrong sign of the exponent", "pow(rope_theta, -2.0 * i / hd)", "pow(rope_theta, 2.0 * i / hd)", False),
    ("body: second norm's gain taken from the first", "rmsnorm_bf16(x, g_mlp[l], d, rms_eps, h);", "rmsnorm_bf16(x, g_attn[l], d, rms_eps, h);", False),
    ("body: residual of the MLP dropped", "linear(wdown[l], d, d_ff, act, proj);\n            for (int i = 0; i < d; ++i) x[i] = round_f32(x[i] + proj[i]);",
     "linear(wdown[l], d, d_ff, act, proj);\n            for (int i = 0; i < d; ++i) x[i] = round_f32(proj[i]);", False),
]


def _run_mutant(args):
    name, old, new, every, tmp = args
    body = name.startswith("body:")
    path = SRC_BODY if body else SRC
    src = open(path).read()
    assert old in src, f"mutant '{name}' no longer matches the oracle's text"
    mutated = src.replace(old, new) if every else src.replace(old, new, 1)
    tag = "".join(ch if ch.isalnum() else "_" for ch in name)
    c_path, so_path = os.path.join(tmp, tag + ".c"), os.path.join(tmp, tag + ".so")
    open(c_path, "w").write(mutated)
    sources = [SRC, c_path] if body else [c_path, SRC_BODY]
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", so_path, *sources, "-lm"], check=True)
    env = dict(os.environ, TABED_ORACLE_LIB=so_path, OMP_NUM_THREADS="2")
    files = [f for f in (BODY_PIN_FILES if body else PIN_FILES) if os.path.exists(os.path.join(ROOT, f))]
    res = subprocess.run([sys.executable, "-m", "pytest", *files, "-x", "-q", "-p", "no:cacheprovider"],
                         cwd=ROOT, env=env, capture_output=True, text=True)
    return name, res.returncode


def test_every_planted_mistake_is_caught_by_a_pin(tmp_path):
    jobs = [(n, o, r, e, str(tmp_path)) for n, o, r, e in MUTANTS + BODY_MUTANTS]
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_run_mutant, jobs))
    missed = [name for name, rc in results if rc == 0]
    assert not missed, f"pins passed with these mistakes planted: {missed}"


def test_the_unmodified_copy_passes(tmp_path):
    """The harness itself: an unmodified copy of the oracle, loaded the same way, passes the same pins."""
    so = str(tmp_path / "copy.so")
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", so, SRC, SRC_BODY, "-lm"], check=True)
    env = dict(os.environ, TABED_ORACLE_LIB=so, OMP_NUM_THREADS="2")
    files = [f for f in PIN_FILES + BODY_PIN_FILES if os.path.exists(os.path.join(ROOT, f))]
    res = subprocess.run([sys.executable, "-m", "pytest", *files, "-x", "-q", "-p", "no:cacheprovider"],
                         cwd=ROOT, env=env, capture_output=True, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
