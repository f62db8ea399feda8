"""ctypes front end of the plain CPU oracle (oracle/tabed_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT: only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import this package.  It shares nothing with
the HIP library; it works on numpy host arrays only.

The arithmetic lives in the C file; this module only marshals arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tabed_oracle.c")
_SRC_BODY = os.path.join(_HERE, "tabed_body_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

FLAG_ACCEPT_MARGIN = 1
FLAG_SAMPLE_MARGIN = 2
FLAG_DEGENERATE = 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math: summation order is part of the definition)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_BODY))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, _SRC_BODY, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        # TABED_ORACLE_LIB: a test that plants mistakes in a COPY of the C file points this module at the copy's
        # build, to show that the pins catch them
        override = os.environ.get("TABED_ORACLE_LIB")
        if override:
            _lib = C.CDLL(override)
        else:
            build()
            _lib = C.CDLL(_LIB)
        _lib.oracle_uniform.restype = C.c_float
        _lib.oracle_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int]
        _lib.oracle_speedup.restype = C.c_double
        _lib.oracle_speedup.argtypes = [C.c_double] * 3
        _lib.oracle_softmax.restype = C.c_double
        _lib.oracle_kl.restype = C.c_double
        _lib.oracle_tvd.restype = C.c_double
        _lib.oracle_argmax.restype = C.c_int
        _lib.oracle_sample_cdf.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def threads() -> int:
    """Number of OpenMP threads the oracle's parallel loops use."""
    omp = C.CDLL("libgomp.so.1")
    omp.omp_get_max_threads.restype = C.c_int
    return int(omp.omp_get_max_threads())


def set_threads(count: int) -> None:
    """Number of OpenMP threads for the calls that follow (timing the oracle on one core and on all of them)."""
    omp = C.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(C.c_int(int(count)))


# ---------------------------------------------------------------- primitives
def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def uniform(seed, rnd, b, pos, word):
    return float(lib().oracle_uniform(seed, rnd, b, pos, word))


def speedup(block_eff, gamma, tq_over_tp):
    return float(lib().oracle_speedup(block_eff, gamma, tq_over_tp))


def lm_head(W, H, w_dtype):
    """W [V,d], H [M,d]: fp32 arrays (w_dtype 0) or uint16 bf16 bit patterns (w_dtype 1)."""
    V, d = W.shape
    M = H.shape[0]
    assert H.shape[1] == d
    want = np.float32 if w_dtype == 0 else np.uint16
    W = np.ascontiguousarray(W, dtype=want)
    H = np.ascontiguousarray(H, dtype=want)
    L = np.empty((M, V), dtype=np.float32)
    lib().oracle_lm_head(M, d, V, w_dtype, _p(W), _p(H), _p(L))
    return L


def softmax(logits, T_eff=1.0):
    x = _f32(logits)
    V = x.shape[0]
    p = np.empty(V, dtype=np.float64)
    logp = np.empty(V, dtype=np.float64)
    lse = lib().oracle_softmax(_p(x), V, C.c_double(T_eff), _p(p), _p(logp))
    return p, logp, float(lse)


def ensemble(q, w):
    q = _f64(q)
    n, V = q.shape
    w = _f32(w)
    out = np.empty(V, dtype=np.float64)
    lib().oracle_ensemble(n, V, _p(q), _p(w), _p(out))
    return out


def argmax(f):
    f = _f64(f)
    flag = C.c_uint32(0)
    v = lib().oracle_argmax(_p(f), f.shape[0], C.byref(flag))
    return int(v), int(flag.value)


def sample_cdf(f, u):
    f = _f64(f)
    flag = C.c_uint32(0)
    v = lib().oracle_sample_cdf(_p(f), f.shape[0], C.c_double(u), C.byref(flag))
    return int(v), int(flag.value)


def kl(p, logp, logq):
    p, logp, logq = _f64(p), _f64(logp), _f64(logq)
    return float(lib().oracle_kl(_p(p), _p(logp), _p(logq), p.shape[0]))


def tvd(p, q):
    p, q = _f64(p), _f64(q)
    return float(lib().oracle_tvd(_p(p), _p(q), p.shape[0]))


# ---------------------------------------------------------------- the three calls
def draft_step(*, V, d, n, B, gamma, w_dtype, seed, rnd, pos, W, H, weights, temperature,
               draft_logits, draft_lse, draft_tokens, draft_q, flags, u_draft=None):
    """Alg. 1 (loop body: draft forward, W-Avg, Sample) at in-block position `pos`; writes slot/column `pos` of the outputs in place."""
    assert draft_logits.dtype == np.float32 and draft_logits.shape == (gamma, B, n, V)
    assert draft_lse.dtype == np.float64 and draft_lse.shape == (gamma, B, n)
    assert draft_tokens.dtype == np.int32 and draft_tokens.shape == (B, gamma)
    assert draft_q.dtype == np.float32 and draft_q.shape == (B, gamma)
    assert flags.dtype == np.uint8 and flags.shape == (B, gamma)
    want = np.float32 if w_dtype == 0 else np.uint16
    W = np.ascontiguousarray(W, dtype=want)
    H = np.ascontiguousarray(H, dtype=want)
    assert W.shape == (V, d) and H.shape == (B, n, d)
    weights = _f32(weights)
    temperature = _f32(temperature)
    u = None if u_draft is None else _f32(u_draft)
    lib().oracle_draft_step(V, d, n, B, gamma, w_dtype, C.c_uint64(seed), C.c_uint64(rnd), pos,
                            _p(W), _p(H), _p(weights), _p(temperature), _p(u),
                            _p(draft_logits), _p(draft_lse), _p(draft_tokens), _p(draft_q), _p(flags))


GRID_CANDIDATES = 11


def dev_width(n, policy):
    """Width of one distance vector: n per-draft distances, or the 11 candidate mixtures of the two-draft grid policy."""
    return GRID_CANDIDATES if policy == 2 else n


def verify(*, V, n, B, gamma, distance, seed, rnd, target_logits, draft_logits, draft_tokens,
           draft_q, weights, temperature, u_acc=None, u_res=None, n_cand=0):
    """Sec. 3 items 2-3 plus per-position distances; returns a dict of fresh output arrays."""
    assert n_cand in (0, GRID_CANDIDATES) and (n_cand == 0 or n == 2)
    target_logits = _f32(target_logits)
    draft_logits = _f32(draft_logits)
    assert target_logits.shape == (B, gamma + 1, V) and draft_logits.shape == (gamma, B, n, V)
    draft_tokens = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    draft_q = _f32(draft_q)
    weights = _f32(weights)
    temperature = _f32(temperature)
    ua = None if u_acc is None else _f32(u_acc)
    ur = None if u_res is None else _f32(u_res)
    out = dict(
        accept_len=np.zeros(B, dtype=np.int32),
        out_tokens=np.full((B, gamma + 1), -1, dtype=np.int32),
        dev=np.zeros((B, gamma, n_cand if n_cand else n), dtype=np.float32),
        n_valid=np.zeros(B, dtype=np.int32),
        flags=np.zeros((B, gamma + 1), dtype=np.uint8),
    )
    lib().oracle_verify(V, n, B, gamma, distance, n_cand, C.c_uint64(seed), C.c_uint64(rnd),
                        _p(target_logits), _p(draft_logits), _p(draft_tokens), _p(draft_q),
                        _p(weights), _p(temperature), _p(ua), _p(ur),
                        _p(out["accept_len"]), _p(out["out_tokens"]), _p(out["dev"]),
                        _p(out["n_valid"]), _p(out["flags"]))
    return out


def update_weights(*, n, B, gamma, h, policy, tau_w, eps, dev, n_valid, ring, ring_head, ring_count, seed=0, rnd=0):
    """Alg. 1 (weight-selection step) (App. B.2 policy); ring state is updated in place; returns weights [B,n]."""
    assert ring.dtype == np.float32 and ring.shape == (B, max(h, 1), dev_width(n, policy))   # h = 0: window ALL
    assert policy != 2 or n == 2
    assert ring_head.dtype == np.int32 and ring_count.dtype == np.int32
    d_ = None if dev is None else _f32(dev)
    nv = None if n_valid is None else np.ascontiguousarray(n_valid, dtype=np.int32)
    w = np.empty((B, n), dtype=np.float32)
    lib().oracle_update_weights(n, B, gamma, h, policy, C.c_double(tau_w), C.c_double(eps),
                                C.c_uint64(seed), C.c_uint64(rnd),
                                _p(d_), _p(nv), _p(ring), _p(ring_head), _p(ring_count), _p(w))
    return w


# ---------------------------------------------------------------- token tree (Sec. 6.1)
SIB_STRIDE = 65536


def draft_siblings(*, V, n, B, gamma, width, seed, rnd, pos, draft_logits, draft_tokens, weights, temperature,
                   sib_tokens, sib_q, sib_flags, u_sib=None):
    """The width-1 sibling candidates of position `pos`, from the ensembled distribution of that position
    (draft_logits slot pos as written by draft_step); writes entries (b, pos, :) of the sib_* arrays in place."""
    S = width - 1
    assert draft_logits.dtype == np.float32 and draft_logits.shape == (gamma, B, n, V)
    assert sib_tokens.dtype == np.int32 and sib_tokens.shape == (B, gamma, S)
    assert sib_q.dtype == np.float32 and sib_q.shape == (B, gamma, S)
    assert sib_flags.dtype == np.uint8 and sib_flags.shape == (B, gamma, S)
    draft_tokens = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    weights, temperature = _f32(weights), _f32(temperature)
    u = None if u_sib is None else _f32(u_sib)
    lib().oracle_draft_siblings(V, n, B, gamma, width, C.c_uint64(seed), C.c_uint64(rnd), pos,
                                _p(draft_logits), _p(draft_tokens), _p(weights), _p(temperature), _p(u),
                                _p(sib_tokens), _p(sib_q), _p(sib_flags))


def verify_tree(*, V, n, B, gamma, width, distance, seed, rnd, target_logits, leaf_logits, draft_logits, draft_tokens,
                draft_q, sib_tokens, sib_q, weights, temperature, u_acc=None, u_res=None, u_acc_sib=None):
    """Verification of a width-`width` token tree; returns a dict of fresh output arrays (those of verify plus
    leaf [B] and n_out [B])."""
    S = width - 1
    assert distance in (0, 1), "hard labels are defined for the chain only"
    target_logits, draft_logits = _f32(target_logits), _f32(draft_logits)
    leaf_logits = _f32(leaf_logits)
    assert target_logits.shape == (B, gamma + 1, V) and draft_logits.shape == (gamma, B, n, V)
    assert leaf_logits.shape == (B, gamma, S, V)
    draft_tokens = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    sib_tokens = np.ascontiguousarray(sib_tokens, dtype=np.int32)
    draft_q, sib_q, weights, temperature = _f32(draft_q), _f32(sib_q), _f32(weights), _f32(temperature)
    assert sib_tokens.shape == (B, gamma, S) and sib_q.shape == (B, gamma, S)
    ua = None if u_acc is None else _f32(u_acc)
    ur = None if u_res is None else _f32(u_res)
    us = None if u_acc_sib is None else _f32(u_acc_sib)
    out = dict(
        accept_len=np.zeros(B, dtype=np.int32),
        out_tokens=np.full((B, gamma + 1), -1, dtype=np.int32),
        dev=np.zeros((B, gamma, n), dtype=np.float32),
        n_valid=np.zeros(B, dtype=np.int32),
        flags=np.zeros((B, gamma + 1), dtype=np.uint8),
        leaf=np.zeros(B, dtype=np.int32),
        n_out=np.zeros(B, dtype=np.int32),
    )
    lib().oracle_verify_tree(V, n, B, gamma, width, distance, C.c_uint64(seed), C.c_uint64(rnd),
                             _p(target_logits), _p(leaf_logits), _p(draft_logits), _p(draft_tokens), _p(draft_q),
                             _p(sib_tokens), _p(sib_q), _p(weights), _p(temperature), _p(ua), _p(ur), _p(us),
                             _p(out["accept_len"]), _p(out["out_tokens"]), _p(out["dev"]), _p(out["n_valid"]),
                             _p(out["flags"]), _p(out["leaf"]), _p(out["n_out"]))
    return out


# ---------------------------------------------------------------- draft-model body (Sec. 5.1 / Sec. 4.1)
def body_step(*, layers, d, heads, d_ff, V, max_ctx, rope_theta, rms_eps, tokens, ctx_len, weights, kcache, vcache):
    """One decode step of the draft model for M rows; appends to the caches in place, returns H [M,d] (bf16 bits).

    weights: dict with embed [V,d] uint16, g_final [d] float32 and per-layer lists g_attn, wqkv, wo, g_mlp, wgu, wdown
    (bf16 bit patterns as uint16, gains float32).  kcache, vcache: uint16 [layers,M,max_ctx,d]."""
    M = len(tokens)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    ctx_len = np.ascontiguousarray(ctx_len, dtype=np.int32)
    assert kcache.dtype == np.uint16 and kcache.shape == (layers, M, max_ctx, d) and vcache.shape == kcache.shape
    assert weights["embed"].dtype == np.uint16 and weights["embed"].shape == (V, d)

    def ptrs(key, dtype, shape):
        arrs = [np.ascontiguousarray(a, dtype=dtype) for a in weights[key]]
        assert len(arrs) == layers and all(a.shape == shape for a in arrs), key
        return arrs, (C.c_void_p * layers)(*[a.ctypes.data for a in arrs])

    keep = []
    plist = []
    for key, dt, shape in (("g_attn", np.float32, (d,)), ("wqkv", np.uint16, (3 * d, d)), ("wo", np.uint16, (d, d)),
                           ("g_mlp", np.float32, (d,)), ("wgu", np.uint16, (2 * d_ff, d)), ("wdown", np.uint16, (d, d_ff))):
        arrs, arr_p = ptrs(key, dt, shape)
        keep.append(arrs)
        plist.append(arr_p)
    g_final = np.ascontiguousarray(weights["g_final"], dtype=np.float32)
    embed = np.ascontiguousarray(weights["embed"])
    H = np.zeros((M, d), dtype=np.uint16)
    lib().oracle_body_step(layers, d, heads, d_ff, V, max_ctx, C.c_double(rope_theta), C.c_double(rms_eps), M,
                           _p(tokens), _p(ctx_len), _p(embed), plist[0], plist[1], plist[2], plist[3], plist[4], plist[5],
                           _p(g_final), _p(kcache), _p(vcache), _p(H))
    return H
