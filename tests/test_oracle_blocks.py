"""Pins for the oracle's building blocks: each check uses a library routine, a closed form or an
invariant -- never the oracle's own formula retyped."""
import os

import numpy as np
import pytest
import scipy.special as sp
import scipy.stats as st

from paper_2601_20357_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Eq. 1
def test_eq1_speedup_matches_paper_worked_example(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eq1_speedup.txt")) if l.strip() and l[0] != "#"]
    assert rows
    for be, gamma, ratio, printed in rows:
        got = oracle.speedup(float(be), float(gamma), float(ratio))
        assert round(got, 2) == float(printed)


# ------------------------------------------------------------------ LM head
def test_lm_head_matches_library_matmul_fp32(oracle):
    rng = np.random.default_rng(1)
    W = rng.standard_normal((37, 24)).astype(np.float32)
    H = rng.standard_normal((5, 24)).astype(np.float32)
    L = oracle.lm_head(W, H, 0)
    ref = H.astype(np.float64) @ W.astype(np.float64).T        # non-square: a transposed operand fails
    assert L.shape == (5, 37)
    np.testing.assert_allclose(L, ref, rtol=0, atol=1e-6)
    assert np.array_equal(L, ref.astype(np.float32)) or np.max(np.abs(L - ref)) < 6e-7


def test_lm_head_bf16_storage_is_upcast_exactly(oracle):
    rng = np.random.default_rng(2)
    Wb = synth.bf16_bits(rng.standard_normal((19, 16)).astype(np.float32) * 0.02)
    Hb = synth.bf16_bits(rng.standard_normal((3, 16)).astype(np.float32))
    L = oracle.lm_head(Wb, Hb, 1)
    ref = synth.bf16_to_f32(Hb).astype(np.float64) @ synth.bf16_to_f32(Wb).astype(np.float64).T
    np.testing.assert_allclose(L, ref.astype(np.float32), rtol=1e-7, atol=1e-9)
    # against the un-rounded inputs the result stays within the bf16 budget (2e-2 relative to scale)
    assert np.max(np.abs(L - ref)) <= 2e-2 * np.max(np.abs(ref))


def test_lm_head_unit_hidden_returns_a_row_of_W(oracle):
    rng = np.random.default_rng(3)
    W = rng.standard_normal((11, 8)).astype(np.float32)
    for k in range(8):
        H = np.zeros((1, 8), dtype=np.float32)
        H[0, k] = 1.0
        assert np.array_equal(oracle.lm_head(W, H, 0)[0], W[:, k])


def test_bf16_helpers_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], dtype=np.float32)   # 1+2^-8 is a tie -> even
    b = synth.bf16_bits(x)
    back = synth.bf16_to_f32(b)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625)
    assert back[3] == -2.5 and back[4] == 0.0


# ------------------------------------------------------------------ softmax
def test_softmax_matches_library_and_invariants(oracle):
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(501) * 3).astype(np.float32)
    for T in (1.0, 0.7, 2.5):
        p, logp, lse = oracle.softmax(x, T)
        np.testing.assert_allclose(p, sp.softmax(x.astype(np.float64) / T), rtol=1e-12)
        np.testing.assert_allclose(logp, sp.log_softmax(x.astype(np.float64) / T), rtol=0, atol=1e-12)
        assert abs(lse - sp.logsumexp(x.astype(np.float64) / T)) < 1e-12
        assert abs(p.sum() - 1.0) < 1e-12
    # shift invariance (exactly representable shift)
    p0, _, lse0 = oracle.softmax(x, 1.0)
    p1, _, lse1 = oracle.softmax((x.astype(np.float64) + 4.0).astype(np.float32), 1.0)
    np.testing.assert_allclose(p1, p0, rtol=1e-5)
    # huge logits do not overflow
    p2, _, _ = oracle.softmax(np.array([1e4, 1e4 - 1, -1e4], dtype=np.float32), 1.0)
    np.testing.assert_allclose(p2, [1 / (1 + np.exp(-1)), np.exp(-1) / (1 + np.exp(-1)), 0.0], rtol=1e-12)


# ------------------------------------------------------------------ ensemble
def test_ensemble_is_probability_space_average(oracle):
    rng = np.random.default_rng(5)
    q = sp.softmax(rng.standard_normal((3, 40)) * 2, axis=1)
    w = np.array([0.2, 0.5, 0.3], dtype=np.float32)
    e = oracle.ensemble(q, w)
    assert abs(e.sum() - float(w.astype(np.float64).sum())) < 1e-12
    np.testing.assert_allclose(e, np.tensordot(w.astype(np.float64), q, axes=1), rtol=1e-13)
    # one-hot weight selects that draft; equal drafts are independent of w
    for j in range(3):
        onehot = np.zeros(3, dtype=np.float32); onehot[j] = 1
        assert np.array_equal(oracle.ensemble(q, onehot), q[j])
    same = np.repeat(q[:1], 3, axis=0)
    np.testing.assert_allclose(oracle.ensemble(same, w), q[0] * float(w.astype(np.float64).sum()), rtol=1e-13)
    # NOT a logit average: a geometric mixture would differ
    geo = sp.softmax(np.tensordot(w.astype(np.float64), np.log(q), axes=1))
    assert np.max(np.abs(e - geo)) > 1e-3


# ------------------------------------------------------------------ distances
def test_kl_matches_library_closed_form_and_direction(oracle):
    rng = np.random.default_rng(6)
    a = (rng.standard_normal(300) * 2).astype(np.float32)
    b = (rng.standard_normal(300) * 2).astype(np.float32)
    p, logp, _ = oracle.softmax(a)
    q, logq, _ = oracle.softmax(b)
    got = oracle.kl(p, logp, logq)
    assert abs(got - sp.rel_entr(p, q).sum()) < 1e-12
    assert got > 0 and abs(oracle.kl(p, logp, logp)) < 1e-15
    rev = oracle.kl(q, logq, logp)
    assert abs(rev - sp.rel_entr(q, p).sum()) < 1e-12 and abs(rev - got) > 1e-3   # direction matters
    # two-token closed form
    pa, qa = 0.3, 0.6
    p2, lp2, _ = oracle.softmax(np.log(np.array([pa, 1 - pa])).astype(np.float32))
    q2, lq2, _ = oracle.softmax(np.log(np.array([qa, 1 - qa])).astype(np.float32))
    closed = p2[0] * np.log(p2[0] / q2[0]) + p2[1] * np.log(p2[1] / q2[1])
    assert abs(oracle.kl(p2, lp2, lq2) - closed) < 1e-14
    # a token whose target probability underflows contributes nothing
    p3, lp3, _ = oracle.softmax(np.array([0.0, -2000.0], dtype=np.float32))
    q3, lq3, _ = oracle.softmax(np.array([0.0, 0.0], dtype=np.float32))
    assert p3[1] == 0.0 and abs(oracle.kl(p3, lp3, lq3) - np.log(2.0)) < 1e-14


def test_tvd_and_pinsker(oracle):
    rng = np.random.default_rng(7)
    for _ in range(5):
        p, logp, _ = oracle.softmax((rng.standard_normal(64) * 2).astype(np.float32))
        q, logq, _ = oracle.softmax((rng.standard_normal(64) * 2).astype(np.float32))
        t = oracle.tvd(p, q)
        assert abs(t - 0.5 * np.abs(p - q).sum()) < 1e-14
        assert abs(t - (1.0 - np.minimum(p, q).sum())) < 1e-12          # TVD = 1 - overlap
        assert t <= np.sqrt(oracle.kl(p, logp, logq) / 2) + 1e-12       # Pinsker
    assert oracle.tvd(p, p) == 0.0


# ------------------------------------------------------------------ argmax / inverse CDF
def test_argmax_lowest_index_and_tie_flag(oracle):
    v, flag = oracle.argmax(np.array([0.1, 0.4, 0.4, 0.1]))
    assert v == 1 and flag & oracle.FLAG_SAMPLE_MARGIN
    v, flag = oracle.argmax(np.array([0.1, 0.2, 0.6, 0.1]))
    assert v == 2 and flag == 0
    v, flag = oracle.argmax(np.array([0.5, 0.5 * (1 - 5e-7)]))
    assert v == 0 and flag & oracle.FLAG_SAMPLE_MARGIN
    assert oracle.argmax(np.array([1.0]))[1] == 0


def test_sample_cdf_is_the_inverse_cdf(oracle):
    f = np.array([0.125, 0.0, 0.25, 0.5, 0.125])       # dyadic: prefix sums exact
    edges = np.cumsum(f)
    for u in np.linspace(0, 1, 257)[:-1] + 1 / 1024:
        v, flag = oracle.sample_cdf(f, u)
        assert v == int(np.searchsorted(edges, u, side="right")) and f[v] > 0
        assert flag == 0
    # exactly on an edge: prefix must EXCEED u*Z, so the next non-empty bin is taken, and it is flagged
    v, flag = oracle.sample_cdf(f, 0.125)
    assert v == 2 and flag & oracle.FLAG_SAMPLE_MARGIN
    # unnormalised input: Z is computed, not assumed
    assert oracle.sample_cdf(f * 7.0, 0.6)[0] == oracle.sample_cdf(f, 0.6)[0] == 3
    # frequencies over a fine midpoint grid reproduce f
    N = 4096
    toks = [oracle.sample_cdf(f, (i + 0.5) / N)[0] for i in range(N)]
    np.testing.assert_allclose(np.bincount(toks, minlength=5) / N, f, atol=1 / N)
    # all-zero input cannot cross: degenerate flag
    v, flag = oracle.sample_cdf(np.zeros(4), 0.3)
    assert flag & oracle.FLAG_DEGENERATE


# ------------------------------------------------------------------ Philox
_M0, _M1 = 0xD2511F53, 0xCD9E8D57
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK = 0xFFFFFFFF


def _philox_inverse(out, key):
    """Undo the 10 rounds from the definition: each round is a bijection because both multipliers are
    odd (invertible mod 2^32).  Written with Python integers, independent of the C code."""
    i0, i1 = pow(_M0, -1, 1 << 32), pow(_M1, -1, 1 << 32)
    keys = [((key[0] + r * _W0) & _MASK, (key[1] + r * _W1) & _MASK) for r in range(10)]
    c = list(out)
    for r in reversed(range(10)):
        k0, k1 = keys[r]
        c2 = (c[1] * i1) & _MASK                    # out1 = lo(M1*c2)
        c0 = (c[3] * i0) & _MASK                    # out3 = lo(M0*c0)
        c1 = c[0] ^ ((_M1 * c2) >> 32) ^ k0         # out0 = hi(M1*c2)^c1^k0
        c3 = c[2] ^ ((_M0 * c0) >> 32) ^ k1         # out2 = hi(M0*c0)^c3^k1
        c = [c0, c1, c2, c3]
    return c


def test_philox_is_the_keyed_bijection_of_its_definition(oracle):
    rng = np.random.default_rng(8)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, 4)]
        key = [int(x) for x in rng.integers(0, 1 << 32, 2)]
        out = [int(x) for x in oracle.philox4x32_10(ctr, key)]
        assert _philox_inverse(out, key) == ctr
    # avalanche: flipping one counter bit flips about half of the 128 output bits
    flips = []
    for bit in range(0, 128, 7):
        ctr = [0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344]
        a = oracle.philox4x32_10(ctr, [1, 2])
        ctr[bit // 32] ^= 1 << (bit % 32)
        b = oracle.philox4x32_10(ctr, [1, 2])
        flips.append(sum(bin(int(x) ^ int(y)).count("1") for x, y in zip(a, b)))
    assert 50 < np.mean(flips) < 78


def _rocrand_engine(tmp_path):
    """rocRAND's Philox4x32-10 engine, compiled for the host from the library's public header."""
    import ctypes as C
    import shutil
    import subprocess
    src = os.path.join(os.path.dirname(__file__), "rocrand_philox_shim.cpp")
    if shutil.which("g++") is None or not os.path.exists("/opt/rocm/include/rocrand/rocrand_philox4x32_10.h"):
        pytest.skip("g++ or the rocRAND headers are not available")
    so = str(tmp_path / "rocrand_philox_shim.so")
    subprocess.run(["g++", "-O1", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-shared", "-fPIC", "-o", so, src],
                   check=True)
    lib = C.CDLL(so)
    lib.shim_philox_next4.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_void_p]
    lib.shim_philox_next4.restype = None
    return lib


def test_philox_matches_rocrand_engine_word_for_word(oracle, tmp_path):
    """The generator IS Philox4x32-10: raw output words equal those of rocRAND's engine (another author's
    implementation) for 4096 random 64-bit keys and full 128-bit counters, plus counters that carry between
    words.  The library maps seed -> key, offset / 4 -> counter words 0-1, subsequence -> counter words 2-3."""
    import ctypes as C
    lib = _rocrand_engine(tmp_path)
    rng = np.random.default_rng(11)
    cases = [(0, 0, 0), (1, 0, 0), (0, 1, 0), (0, 0, 1), (2 ** 64 - 1, 2 ** 64 - 1, 2 ** 62 - 1), (5, 7, 2 ** 32 - 1),
             (5, 7, 2 ** 32), (5, 2 ** 32, 9), (2 ** 32, 3, 9)]
    cases += [tuple(int(x) for x in (rng.integers(0, 2 ** 64, dtype=np.uint64), rng.integers(0, 2 ** 64, dtype=np.uint64),
                                     rng.integers(0, 2 ** 62, dtype=np.uint64))) for _ in range(4096)]
    out = np.zeros(4, np.uint32)
    for seed, sub, cnt in cases:
        lib.shim_philox_next4(seed, sub, cnt * 4, out.ctypes.data_as(C.c_void_p))
        ours = oracle.philox4x32_10([cnt & _MASK, cnt >> 32, sub & _MASK, sub >> 32], [seed & _MASK, seed >> 32])
        assert np.array_equal(out, ours), (seed, sub, cnt)
    # the method's own keying: key = seed, counter = (round lo, round hi, b, pos); u = (word >> 8) * 2^-24
    for seed, rnd, b, pos in [(0, 0, 0, 0), (0x123456789ABCDEF, (1 << 40) + 5, 63, 15), (7, 3, 2, 1)]:
        lib.shim_philox_next4(seed, b | (pos << 32), rnd * 4, out.ctypes.data_as(C.c_void_p))
        for word in (0, 1):
            assert oracle.uniform(seed, rnd, b, pos, word) == float(np.float32(int(out[word]) >> 8) * np.float32(2.0 ** -24))


def test_uniforms_are_uniform_exact_and_keyed_by_seed_round_b_pos(oracle):
    us = np.array([[oracle.uniform(0, r, b, p, w) for w in (0, 1)]
                   for r in range(40) for b in range(16) for p in range(6)])
    assert us.min() >= 0.0 and us.max() < 1.0
    assert np.all(us * 2 ** 24 == np.round(us * 2 ** 24))        # multiples of 2^-24 ...
    odd = np.mean((us * 2 ** 24).astype(np.int64) % 2 == 1)
    assert 0.45 < odd < 0.55                                     # ... and all 24 bits are used
    assert us.max() > 1 - 2.0 ** -9 or len(us) < 1000            # the top of [0,1) is reachable
    assert st.kstest(us[:, 0], "uniform").pvalue > 1e-3
    assert st.kstest(us[:, 1], "uniform").pvalue > 1e-3
    assert abs(np.corrcoef(us[:, 0], us[:, 1])[0, 1]) < 0.05
    base = oracle.uniform(7, 3, 2, 1, 0)
    assert base == oracle.uniform(7, 3, 2, 1, 0)
    others = [oracle.uniform(8, 3, 2, 1, 0), oracle.uniform(7, 4, 2, 1, 0), oracle.uniform(7, 3, 3, 1, 0),
              oracle.uniform(7, 3, 2, 2, 0), oracle.uniform(7, 3, 2, 1, 1), oracle.uniform(7 + (1 << 32), 3, 2, 1, 0),
              oracle.uniform(7, 3 + (1 << 32), 2, 1, 0)]
    assert all(o != base for o in others)
