"""Thin ctypes binding of libtabed.so: same names as the C ABI in include/tabed.h, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors; torch is used for device memory and streams, nothing else.
Every step of the path runs inside the library's HIP kernels.  There is no fallback: if the library has
not been built, or a call returns an error code, this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtabed.so")

EXPORTS = [
    "tabed_workspace_bytes", "tabed_workspace_init", "tabed_strerror", "tabed_last_hip_error", "tabed_dev_width",
    "tabed_draft_step", "tabed_draft_step_static", "tabed_verify", "tabed_draft_siblings", "tabed_verify_tree", "tabed_update_weights", "tabed_philox_uniforms",
    "tabed_body_workspace_bytes", "tabed_body_workspace_init", "tabed_draft_body_step", "tabed_draft_body_rollback",
    "tabed_prof_enable", "tabed_prof_read", "tabed_prof_reset", "tabed_kernel_name", "tabed_prof_null",
]

FLAG_ACCEPT_MARGIN, FLAG_SAMPLE_MARGIN, FLAG_DEGENERATE = 1, 2, 4
K_LMHEAD, K_SAMPLE, K_STATS, K_RESID, K_WEIGHTS, K_DIST, K_TREE, K_BODY, K_NULL, K_COUNT = 0, 1, 2, 3, 4, 5, 6, 7, 8, 9
BODY_MAX_LAYERS = 16


class TabedCfg(C.Structure):
    """Mirror of `tabed_cfg`."""
    _fields_ = [("V", C.c_int32), ("d", C.c_int32), ("n", C.c_int32), ("B", C.c_int32),
                ("gamma", C.c_int32), ("h", C.c_int32), ("w_dtype", C.c_int32), ("distance", C.c_int32),
                ("policy", C.c_int32), ("tau_w", C.c_float), ("eps", C.c_float), ("seed", C.c_uint64)]


class TabedBodyCfg(C.Structure):
    """Mirror of `tabed_body_cfg`."""
    _fields_ = [("layers", C.c_int32), ("d", C.c_int32), ("heads", C.c_int32), ("d_ff", C.c_int32), ("V", C.c_int32),
                ("max_ctx", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class TabedBodyWeights(C.Structure):
    """Mirror of `tabed_body_weights` (device pointers)."""
    _fields_ = [("embed", C.c_void_p), ("g_final", C.c_void_p)] + [
        (name, C.c_void_p * BODY_MAX_LAYERS) for name in ("g_attn", "wqkv", "wo", "g_mlp", "wgu", "wdown")]


class TabedError(RuntimeError):
    pass


_lib = None


def load():
    """Load libtabed.so; raises if it has not been built (python -m paper_2601_20357_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise TabedError(f"{LIB_PATH} is missing: build it first (python paper_2601_20357_amd/build.py); "
                         "there is no CPU fallback")
    lib = C.CDLL(LIB_PATH)
    vp, u64, i32 = C.c_void_p, C.c_uint64, C.c_int32
    cfgp = C.POINTER(TabedCfg)
    lib.tabed_workspace_bytes.restype = C.c_size_t
    lib.tabed_workspace_bytes.argtypes = [cfgp]
    lib.tabed_dev_width.restype = C.c_int32
    lib.tabed_dev_width.argtypes = [cfgp]
    lib.tabed_workspace_init.restype = C.c_int
    lib.tabed_workspace_init.argtypes = [cfgp, vp, vp]
    lib.tabed_strerror.restype = C.c_char_p
    lib.tabed_strerror.argtypes = [C.c_int]
    lib.tabed_last_hip_error.restype = C.c_int
    lib.tabed_draft_step.restype = C.c_int
    lib.tabed_draft_step.argtypes = [cfgp, vp, u64, i32] + [vp] * 11
    lib.tabed_draft_step_static.restype = C.c_int
    lib.tabed_draft_step_static.argtypes = [cfgp, u64, i32] + [vp] * 11
    lib.tabed_verify.restype = C.c_int
    lib.tabed_verify.argtypes = [cfgp, vp, u64] + [vp] * 19
    lib.tabed_draft_siblings.restype = C.c_int
    lib.tabed_draft_siblings.argtypes = [cfgp, vp, u64, i32, i32] + [vp] * 9
    lib.tabed_verify_tree.restype = C.c_int
    lib.tabed_verify_tree.argtypes = [cfgp, vp, u64, i32] + [vp] * 25
    lib.tabed_update_weights.restype = C.c_int
    lib.tabed_update_weights.argtypes = [cfgp, vp, u64] + [vp] * 7
    lib.tabed_philox_uniforms.restype = C.c_int
    lib.tabed_philox_uniforms.argtypes = [cfgp, u64, vp, vp]
    bcfgp = C.POINTER(TabedBodyCfg)
    lib.tabed_body_workspace_bytes.restype = C.c_size_t
    lib.tabed_body_workspace_bytes.argtypes = [bcfgp, i32]
    lib.tabed_body_workspace_init.restype = C.c_int
    lib.tabed_body_workspace_init.argtypes = [bcfgp, i32, vp, vp]
    lib.tabed_draft_body_step.restype = C.c_int
    lib.tabed_draft_body_step.argtypes = [bcfgp, C.POINTER(TabedBodyWeights), vp, i32, vp, i32, i32] + [vp] * 5
    lib.tabed_draft_body_rollback.restype = C.c_int
    lib.tabed_draft_body_rollback.argtypes = [i32, i32, i32, vp, vp, vp, vp]
    lib.tabed_prof_enable.restype = C.c_int
    lib.tabed_prof_enable.argtypes = [C.c_int]
    lib.tabed_prof_read.restype = C.c_int
    lib.tabed_prof_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.tabed_prof_reset.restype = C.c_int
    lib.tabed_kernel_name.restype = C.c_char_p
    lib.tabed_kernel_name.argtypes = [C.c_int]
    lib.tabed_prof_null.restype = C.c_int
    lib.tabed_prof_null.argtypes = [vp]
    _lib = lib
    return lib


GRID_CANDIDATES = 11


def make_cfg(*, V, d, n, B, gamma, h, w_dtype, distance=0, policy=0, tau_w=1.0, eps=1e-6, seed=0) -> TabedCfg:
    return TabedCfg(V, d, n, B, gamma, h, w_dtype, distance, policy, tau_w, eps, seed)


def _check(rc: int, what: str):
    if rc != 0:
        lib = load()
        msg = lib.tabed_strerror(rc).decode()
        raise TabedError(f"{what}: {msg} (code {rc}, hip error {lib.tabed_last_hip_error()})")


def _ptr(t, dtype=None, numel=None, name="tensor"):
    """Device pointer of a contiguous CUDA tensor (None -> NULL), with dtype / size checks."""
    if t is None:
        return None
    if not t.is_cuda:
        raise TabedError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise TabedError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TabedError(f"{name} must be {dtype}, got {t.dtype}")
    if numel is not None and t.numel() != numel:
        raise TabedError(f"{name} must hold {numel} elements, got {t.numel()}")
    return t.data_ptr()


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def tabed_dev_width(cfg: TabedCfg) -> int:
    """Last dimension of `dev` and `ring`: n, or 11 for the two-draft grid policy; 0 for an invalid cfg."""
    return int(load().tabed_dev_width(C.byref(cfg)))


def tabed_workspace_bytes(cfg: TabedCfg) -> int:
    return int(load().tabed_workspace_bytes(C.byref(cfg)))


def tabed_workspace_init(cfg: TabedCfg, ws, stream=None):
    _check(load().tabed_workspace_init(C.byref(cfg), _ptr(ws, name="ws"), _stream(stream)), "tabed_workspace_init")


def new_workspace(cfg: TabedCfg, device="cuda:0", stream=None):
    """Allocate (torch) and prepare a workspace for cfg."""
    import torch
    nbytes = tabed_workspace_bytes(cfg)
    if nbytes == 0:
        raise TabedError("invalid or unsupported tabed_cfg")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    tabed_workspace_init(cfg, ws, stream)
    return ws


def _store_dtype(cfg):
    import torch
    return torch.float32 if cfg.w_dtype == 0 else torch.bfloat16


def tabed_draft_step(cfg, ws, rnd, pos, W, H, weights, temperature, draft_logits, draft_lse, draft_tokens,
                     draft_q, flags, u_draft=None, stream=None):
    import torch
    V, d, n, B, g = cfg.V, cfg.d, cfg.n, cfg.B, cfg.gamma
    sd = _store_dtype(cfg)
    rc = load().tabed_draft_step(
        C.byref(cfg), _ptr(ws, torch.uint8, name="ws"), rnd, pos,
        _ptr(W, sd, V * d, "W"), _ptr(H, sd, B * n * d, "H"),
        _ptr(weights, torch.float32, B * n, "weights"), _ptr(temperature, torch.float32, B, "temperature"),
        _ptr(u_draft, torch.float32, B * g, "u_draft"),
        _ptr(draft_logits, torch.float32, g * B * n * V, "draft_logits"),
        _ptr(draft_lse, torch.float64, g * B * n, "draft_lse"),
        _ptr(draft_tokens, torch.int32, B * g, "draft_tokens"), _ptr(draft_q, torch.float32, B * g, "draft_q"),
        _ptr(flags, torch.uint8, B * g, "flags"), _stream(stream))
    _check(rc, "tabed_draft_step")


STATIC_SCRATCH_BYTES = 8 << 20
ETOOBIG = -7


def tabed_draft_step_static(cfg, rnd, pos, W, H, weights, temperature, draft_logits, draft_lse, draft_tokens,
                            draft_q, flags, u_draft=None, stream=None):
    """tabed_draft_step on the library's built-in scratch buffer (no workspace argument, nothing allocated)."""
    import torch
    V, d, n, B, g = cfg.V, cfg.d, cfg.n, cfg.B, cfg.gamma
    sd = _store_dtype(cfg)
    rc = load().tabed_draft_step_static(
        C.byref(cfg), rnd, pos,
        _ptr(W, sd, V * d, "W"), _ptr(H, sd, B * n * d, "H"),
        _ptr(weights, torch.float32, B * n, "weights"), _ptr(temperature, torch.float32, B, "temperature"),
        _ptr(u_draft, torch.float32, B * g, "u_draft"),
        _ptr(draft_logits, torch.float32, g * B * n * V, "draft_logits"),
        _ptr(draft_lse, torch.float64, g * B * n, "draft_lse"),
        _ptr(draft_tokens, torch.int32, B * g, "draft_tokens"), _ptr(draft_q, torch.float32, B * g, "draft_q"),
        _ptr(flags, torch.uint8, B * g, "flags"), _stream(stream))
    _check(rc, "tabed_draft_step_static")


def tabed_verify(cfg, ws, rnd, target_logits, draft_logits, draft_lse, draft_tokens, draft_q, weights, temperature,
                 accept_len, out_tokens, dev, n_valid, flags, u_acc=None, u_res=None, ring=None, ring_head=None,
                 ring_count=None, next_weights=None, stream=None):
    import torch
    V, n, B, g = cfg.V, cfg.n, cfg.B, cfg.gamma
    rc = load().tabed_verify(
        C.byref(cfg), _ptr(ws, torch.uint8, name="ws"), rnd,
        _ptr(target_logits, torch.float32, B * (g + 1) * V, "target_logits"),
        _ptr(draft_logits, torch.float32, g * B * n * V, "draft_logits"),
        _ptr(draft_lse, torch.float64, g * B * n, "draft_lse"),
        _ptr(draft_tokens, torch.int32, B * g, "draft_tokens"), _ptr(draft_q, torch.float32, B * g, "draft_q"),
        _ptr(weights, torch.float32, B * n, "weights"), _ptr(temperature, torch.float32, B, "temperature"),
        _ptr(u_acc, torch.float32, B * g, "u_acc"), _ptr(u_res, torch.float32, B, "u_res"),
        _ptr(accept_len, torch.int32, B, "accept_len"), _ptr(out_tokens, torch.int32, B * (g + 1), "out_tokens"),
        _ptr(dev, torch.float32, B * g * tabed_dev_width(cfg), "dev"), _ptr(n_valid, torch.int32, B, "n_valid"),
        _ptr(flags, torch.uint8, B * (g + 1), "flags"),
        _ptr(ring, torch.float32, B * max(cfg.h, 1) * tabed_dev_width(cfg), "ring"),
        _ptr(ring_head, torch.int32, B, "ring_head"), _ptr(ring_count, torch.int32, B, "ring_count"),
        _ptr(next_weights, torch.float32, B * n, "next_weights"), _stream(stream))
    _check(rc, "tabed_verify")


MAX_TREE_WIDTH = 3
SIBLING_STRIDE = 65536


def tabed_draft_siblings(cfg, ws, rnd, pos, tree_width, draft_logits, draft_tokens, weights, temperature, sib_tokens,
                         sib_q, sib_flags, u_sib=None, stream=None):
    import torch
    V, n, B, g = cfg.V, cfg.n, cfg.B, cfg.gamma
    S = tree_width - 1
    rc = load().tabed_draft_siblings(
        C.byref(cfg), _ptr(ws, torch.uint8, name="ws"), rnd, pos, tree_width,
        _ptr(draft_logits, torch.float32, g * B * n * V, "draft_logits"),
        _ptr(draft_tokens, torch.int32, B * g, "draft_tokens"),
        _ptr(weights, torch.float32, B * n, "weights"), _ptr(temperature, torch.float32, B, "temperature"),
        _ptr(u_sib, torch.float32, B * g * S, "u_sib"),
        _ptr(sib_tokens, torch.int32, B * g * S, "sib_tokens"), _ptr(sib_q, torch.float32, B * g * S, "sib_q"),
        _ptr(sib_flags, torch.uint8, B * g * S, "sib_flags"), _stream(stream))
    _check(rc, "tabed_draft_siblings")


def tabed_verify_tree(cfg, ws, rnd, tree_width, target_logits, leaf_logits, draft_logits, draft_lse, draft_tokens,
                      draft_q, sib_tokens, sib_q, weights, temperature, accept_len, out_tokens, dev, n_valid, flags,
                      leaf, n_out, u_acc=None, u_res=None, u_acc_sib=None, ring=None, ring_head=None, ring_count=None,
                      next_weights=None, stream=None):
    import torch
    V, n, B, g = cfg.V, cfg.n, cfg.B, cfg.gamma
    S = tree_width - 1
    dw = tabed_dev_width(cfg)
    rc = load().tabed_verify_tree(
        C.byref(cfg), _ptr(ws, torch.uint8, name="ws"), rnd, tree_width,
        _ptr(target_logits, torch.float32, B * (g + 1) * V, "target_logits"),
        _ptr(leaf_logits, torch.float32, B * g * S * V, "leaf_logits") if S else None,
        _ptr(draft_logits, torch.float32, g * B * n * V, "draft_logits"),
        _ptr(draft_lse, torch.float64, g * B * n, "draft_lse"),
        _ptr(draft_tokens, torch.int32, B * g, "draft_tokens"), _ptr(draft_q, torch.float32, B * g, "draft_q"),
        _ptr(sib_tokens, torch.int32, B * g * S, "sib_tokens") if S else None,
        _ptr(sib_q, torch.float32, B * g * S, "sib_q") if S else None,
        _ptr(weights, torch.float32, B * n, "weights"), _ptr(temperature, torch.float32, B, "temperature"),
        _ptr(u_acc, torch.float32, B * g, "u_acc"), _ptr(u_res, torch.float32, B, "u_res"),
        _ptr(u_acc_sib, torch.float32, B * g * S, "u_acc_sib") if S else None,
        _ptr(accept_len, torch.int32, B, "accept_len"), _ptr(out_tokens, torch.int32, B * (g + 1), "out_tokens"),
        _ptr(dev, torch.float32, B * g * dw, "dev"), _ptr(n_valid, torch.int32, B, "n_valid"),
        _ptr(flags, torch.uint8, B * (g + 1), "flags"), _ptr(leaf, torch.int32, B, "leaf"),
        _ptr(n_out, torch.int32, B, "n_out"),
        _ptr(ring, torch.float32, B * max(cfg.h, 1) * dw, "ring"),
        _ptr(ring_head, torch.int32, B, "ring_head"), _ptr(ring_count, torch.int32, B, "ring_count"),
        _ptr(next_weights, torch.float32, B * n, "next_weights"), _stream(stream))
    _check(rc, "tabed_verify_tree")


def tabed_update_weights(cfg, ws, rnd, dev, n_valid, ring, ring_head, ring_count, weights, stream=None):
    import torch
    n, B, g, h = cfg.n, cfg.B, cfg.gamma, cfg.h
    dw = tabed_dev_width(cfg)
    rc = load().tabed_update_weights(
        C.byref(cfg), _ptr(ws, name="ws"), rnd,
        _ptr(dev, torch.float32, B * g * dw, "dev"), _ptr(n_valid, torch.int32, B, "n_valid"),
        _ptr(ring, torch.float32, B * max(h, 1) * dw, "ring"), _ptr(ring_head, torch.int32, B, "ring_head"),
        _ptr(ring_count, torch.int32, B, "ring_count"), _ptr(weights, torch.float32, B * n, "weights"),
        _stream(stream))
    _check(rc, "tabed_update_weights")


def make_body_cfg(*, layers, d, heads, d_ff, V, max_ctx, rope_theta=1e4, rms_eps=1e-5) -> TabedBodyCfg:
    return TabedBodyCfg(layers, d, heads, d_ff, V, max_ctx, rope_theta, rms_eps)


def make_body_weights(bcfg: TabedBodyCfg, tensors: dict) -> TabedBodyWeights:
    """Pointer table over device tensors: embed [V,d] and the per-layer lists wqkv [3d,d], wo [d,d], wgu [2 d_ff,d],
    wdown [d,d_ff] as bf16 (or their bit patterns as int16 / uint16), gains g_attn, g_mlp (lists) and g_final as fp32.
    The caller keeps `tensors` alive while the table is in use."""
    import torch
    two_byte = (torch.bfloat16, torch.int16, torch.uint16)
    d, ff, L = bcfg.d, bcfg.d_ff, bcfg.layers

    def mat(t, numel, name):
        if t.dtype not in two_byte:
            raise TabedError(f"{name} must hold bf16 values, got {t.dtype}")
        return _ptr(t, None, numel, name)

    w = TabedBodyWeights()
    w.embed = mat(tensors["embed"], bcfg.V * d, "embed")
    w.g_final = _ptr(tensors["g_final"], torch.float32, d, "g_final")
    for key, numel in (("wqkv", 3 * d * d), ("wo", d * d), ("wgu", 2 * ff * d), ("wdown", d * ff)):
        if len(tensors[key]) != L:
            raise TabedError(f"{key} must list {L} layers")
        for l in range(L):
            getattr(w, key)[l] = mat(tensors[key][l], numel, f"{key}[{l}]")
    for key in ("g_attn", "g_mlp"):
        if len(tensors[key]) != L:
            raise TabedError(f"{key} must list {L} layers")
        for l in range(L):
            getattr(w, key)[l] = _ptr(tensors[key][l], torch.float32, d, f"{key}[{l}]")
    return w


def tabed_body_workspace_bytes(bcfg: TabedBodyCfg, rows: int) -> int:
    return int(load().tabed_body_workspace_bytes(C.byref(bcfg), rows))


def tabed_body_workspace_init(bcfg, rows, ws, stream=None):
    import torch
    need = tabed_body_workspace_bytes(bcfg, rows)
    if need == 0:
        raise TabedError("tabed_body_workspace_init: invalid configuration")
    if ws.numel() * ws.element_size() < need:
        raise TabedError(f"body workspace holds {ws.numel() * ws.element_size()} bytes, {need} needed")
    _check(load().tabed_body_workspace_init(C.byref(bcfg), rows, _ptr(ws, torch.uint8, name="ws"), _stream(stream)),
           "tabed_body_workspace_init")


def tabed_draft_body_step(bcfg, weights, ws, rows, token_src, token_stride, rows_per_token, ctx_len, kcache, vcache, H,
                          stream=None):
    """token_src: int32 tensor, or a (tensor, element offset) pair for a view into draft_tokens."""
    import torch
    if isinstance(token_src, tuple):
        base, off = token_src
        need = off + ((rows - 1) // rows_per_token) * token_stride + 1
        if base.dtype != torch.int32 or not base.is_cuda or not base.is_contiguous() or base.numel() < need or off < 0:
            raise TabedError("token_src must be a contiguous int32 GPU tensor covering every token read")
        tok_ptr = base.data_ptr() + 4 * off
    else:
        need = ((rows - 1) // rows_per_token) * token_stride + 1
        if token_src.numel() < need:
            raise TabedError(f"token_src must hold {need} elements, got {token_src.numel()}")
        tok_ptr = _ptr(token_src, torch.int32, None, "token_src")
    if ws.numel() * ws.element_size() < tabed_body_workspace_bytes(bcfg, rows):
        raise TabedError("body workspace too small")
    two_byte = (torch.bfloat16, torch.int16, torch.uint16)
    for t, name in ((kcache, "kcache"), (vcache, "vcache"), (H, "H")):
        if t.dtype not in two_byte:
            raise TabedError(f"{name} must hold bf16 values, got {t.dtype}")
    cache_numel = bcfg.layers * rows * bcfg.max_ctx * bcfg.d
    rc = load().tabed_draft_body_step(
        C.byref(bcfg), C.byref(weights), _ptr(ws, torch.uint8, name="ws"), rows, tok_ptr, token_stride, rows_per_token,
        _ptr(ctx_len, torch.int32, rows, "ctx_len"), _ptr(kcache, None, cache_numel, "kcache"),
        _ptr(vcache, None, cache_numel, "vcache"), _ptr(H, None, rows * bcfg.d, "H"), _stream(stream))
    _check(rc, "tabed_draft_body_step")


def tabed_draft_body_rollback(rows, rows_per_seq, gamma, ctx_base, accept_len, ctx_len, stream=None):
    import torch
    nseq = (rows + rows_per_seq - 1) // rows_per_seq
    rc = load().tabed_draft_body_rollback(
        rows, rows_per_seq, gamma, _ptr(ctx_base, torch.int32, rows, "ctx_base"),
        _ptr(accept_len, torch.int32, nseq, "accept_len"), _ptr(ctx_len, torch.int32, rows, "ctx_len"), _stream(stream))
    _check(rc, "tabed_draft_body_rollback")


def tabed_philox_uniforms(cfg, rnd, out, stream=None):
    import torch
    rc = load().tabed_philox_uniforms(C.byref(cfg), rnd, _ptr(out, torch.float32, cfg.B * (cfg.gamma + 1) * 2, "out"),
                                      _stream(stream))
    _check(rc, "tabed_philox_uniforms")


def tabed_prof_enable(on: bool):
    _check(load().tabed_prof_enable(1 if on else 0), "tabed_prof_enable")


def tabed_prof_reset():
    _check(load().tabed_prof_reset(), "tabed_prof_reset")


def tabed_prof_read(kernel_id: int):
    """(total milliseconds, launches) of one kernel since the last reset; waits for its events."""
    ms, cnt = C.c_double(0), C.c_int64(0)
    _check(load().tabed_prof_read(kernel_id, C.byref(ms), C.byref(cnt)), "tabed_prof_read")
    return ms.value, cnt.value


def tabed_prof_null(stream=None):
    _check(load().tabed_prof_null(_stream(stream)), "tabed_prof_null")


def tabed_kernel_name(kernel_id: int) -> str:
    return load().tabed_kernel_name(kernel_id).decode()


class PreparedCall:
    """A C-ABI call with its arguments already converted to ctypes, for launch loops where the per-call
    tensor checks would cost more than the launch.  Built by RoundBuffers.prepare_*; checks happen once."""

    __slots__ = ("fn", "args", "what", "round_arg")

    def __init__(self, fn, args, what, round_arg=None):
        self.fn, self.args, self.what, self.round_arg = fn, args, what, round_arg

    def set_round(self, rnd: int):
        """Change the SD round number (the Philox counter) the next call passes."""
        if self.round_arg is not None:
            self.round_arg.value = rnd

    def __call__(self):
        rc = self.fn(*self.args)
        if rc != 0:
            _check(rc, self.what)


class BodyBuffers:
    """Device buffers of the draft-model body for `rows` rows (allocation only; no arithmetic here): weight table,
    scratch, key / value caches, positions and the hidden states H the LM head reads."""

    def __init__(self, bcfg: TabedBodyCfg, rows: int, tensors: dict, device="cuda:0"):
        import torch
        self.cfg, self.rows, self.tensors = bcfg, rows, tensors
        self.table = make_body_weights(bcfg, tensors)
        need = tabed_body_workspace_bytes(bcfg, rows)
        if need == 0:
            raise TabedError("invalid body configuration")
        self.ws = torch.empty(need, dtype=torch.uint8, device=device)
        tabed_body_workspace_init(bcfg, rows, self.ws)
        self.kcache = torch.zeros((bcfg.layers, rows, bcfg.max_ctx, bcfg.d), dtype=torch.bfloat16, device=device)
        self.vcache = torch.zeros_like(self.kcache)
        self.ctx_len = torch.zeros(rows, dtype=torch.int32, device=device)
        self.ctx_base = torch.zeros(rows, dtype=torch.int32, device=device)
        self.H = torch.zeros((rows, bcfg.d), dtype=torch.bfloat16, device=device)

    def prepare_step(self, token_src, token_offset, token_stride, rows_per_token, stream=None) -> PreparedCall:
        import torch
        need = token_offset + ((self.rows - 1) // rows_per_token) * token_stride + 1
        if token_src.dtype != torch.int32 or not token_src.is_cuda or not token_src.is_contiguous() or token_src.numel() < need:
            raise TabedError("token_src must be a contiguous int32 GPU tensor covering every token read")
        vp = C.c_void_p
        args = [C.byref(self.cfg), C.byref(self.table), vp(self.ws.data_ptr()), C.c_int32(self.rows),
                vp(token_src.data_ptr() + 4 * token_offset), C.c_int32(token_stride), C.c_int32(rows_per_token),
                vp(self.ctx_len.data_ptr()), vp(self.kcache.data_ptr()), vp(self.vcache.data_ptr()), vp(self.H.data_ptr()),
                vp(_stream(stream))]
        return PreparedCall(load().tabed_draft_body_step, args, "tabed_draft_body_step")

    def prepare_rollback(self, rows_per_seq, gamma, accept_len, stream=None) -> PreparedCall:
        import torch
        vp = C.c_void_p
        nseq = (self.rows + rows_per_seq - 1) // rows_per_seq
        args = [C.c_int32(self.rows), C.c_int32(rows_per_seq), C.c_int32(gamma), vp(self.ctx_base.data_ptr()),
                vp(_ptr(accept_len, torch.int32, nseq, "accept_len")), vp(self.ctx_len.data_ptr()), vp(_stream(stream))]
        return PreparedCall(load().tabed_draft_body_rollback, args, "tabed_draft_body_rollback")


class RoundBuffers:
    """Device buffers one sequence batch needs across rounds (allocation only; no arithmetic here)."""

    def __init__(self, cfg: TabedCfg, device="cuda:0"):
        import torch
        V, n, B, g, h = cfg.V, cfg.n, cfg.B, cfg.gamma, cfg.h
        z = lambda shape, dt: torch.zeros(shape, dtype=dt, device=device)
        self.cfg = cfg
        self.ws = new_workspace(cfg, device)
        dw = tabed_dev_width(cfg)
        self.weights = z((B, n), torch.float32)
        self.ring = z((B, max(h, 1), dw), torch.float32)      # h = 0: window ALL keeps one running sum
        self.ring_head = z((B,), torch.int32)
        self.ring_count = z((B,), torch.int32)
        self.draft_logits = z((g, B, n, V), torch.float32)
        self.draft_lse = z((g, B, n), torch.float64)
        self.draft_tokens = z((B, g), torch.int32)
        self.draft_q = z((B, g), torch.float32)
        self.draft_flags = z((B, g), torch.uint8)
        self.accept_len = z((B,), torch.int32)
        self.out_tokens = z((B, g + 1), torch.int32)
        self.dev = z((B, g, dw), torch.float32)
        self.n_valid = z((B,), torch.int32)
        self.verify_flags = z((B, g + 1), torch.uint8)

    # ---- token tree: sibling candidates and the walk's extra outputs
    def enable_tree(self, width: int):
        import torch
        c = self.cfg
        S = width - 1
        dev = self.weights.device
        self.tree_width = width
        self.sib_tokens = torch.zeros((c.B, c.gamma, S), dtype=torch.int32, device=dev)
        self.sib_q = torch.zeros((c.B, c.gamma, S), dtype=torch.float32, device=dev)
        self.sib_flags = torch.zeros((c.B, c.gamma, S), dtype=torch.uint8, device=dev)
        self.leaf = torch.zeros((c.B,), dtype=torch.int32, device=dev)
        self.n_out = torch.zeros((c.B,), dtype=torch.int32, device=dev)

    def prepare_draft_siblings(self, rnd, pos, temperature, stream=None) -> "PreparedCall":
        import torch
        c = self.cfg
        vp = C.c_void_p
        args = [C.byref(c), vp(self.ws.data_ptr()), C.c_uint64(rnd), C.c_int32(pos), C.c_int32(self.tree_width),
                vp(self.draft_logits.data_ptr()), vp(self.draft_tokens.data_ptr()), vp(self.weights.data_ptr()),
                vp(_ptr(temperature, torch.float32, c.B, "temperature")), vp(None),
                vp(self.sib_tokens.data_ptr()), vp(self.sib_q.data_ptr()), vp(self.sib_flags.data_ptr()),
                vp(_stream(stream))]
        return PreparedCall(load().tabed_draft_siblings, args, "tabed_draft_siblings", args[2])

    def prepare_verify_tree(self, rnd, target_logits, leaf_logits, temperature, stream=None) -> "PreparedCall":
        """The window update stays a separate call here (next_weights may not alias weights in tabed_verify_tree)."""
        import torch
        c = self.cfg
        vp = C.c_void_p
        S = self.tree_width - 1
        args = [C.byref(c), vp(self.ws.data_ptr()), C.c_uint64(rnd), C.c_int32(self.tree_width),
                vp(_ptr(target_logits, torch.float32, c.B * (c.gamma + 1) * c.V, "target_logits")),
                vp(_ptr(leaf_logits, torch.float32, c.B * c.gamma * S * c.V, "leaf_logits")),
                vp(self.draft_logits.data_ptr()), vp(self.draft_lse.data_ptr()), vp(self.draft_tokens.data_ptr()),
                vp(self.draft_q.data_ptr()), vp(self.sib_tokens.data_ptr()), vp(self.sib_q.data_ptr()),
                vp(self.weights.data_ptr()), vp(_ptr(temperature, torch.float32, c.B, "temperature")),
                vp(None), vp(None), vp(None),
                vp(self.accept_len.data_ptr()), vp(self.out_tokens.data_ptr()), vp(self.dev.data_ptr()),
                vp(self.n_valid.data_ptr()), vp(self.verify_flags.data_ptr()), vp(self.leaf.data_ptr()),
                vp(self.n_out.data_ptr()), vp(None), vp(None), vp(None), vp(None), vp(_stream(stream))]
        return PreparedCall(load().tabed_verify_tree, args, "tabed_verify_tree", args[2])

    # ---- the same three calls with arguments converted once (hot loops)
    def prepare_update_weights(self, first: bool, rnd=0, stream=None) -> PreparedCall:
        import torch
        c = self.cfg
        vp = C.c_void_p
        args = [C.byref(c), vp(self.ws.data_ptr()), C.c_uint64(rnd),
                vp(None if first else self.dev.data_ptr()), vp(None if first else self.n_valid.data_ptr()),
                vp(self.ring.data_ptr()), vp(self.ring_head.data_ptr()), vp(self.ring_count.data_ptr()),
                vp(self.weights.data_ptr()), vp(_stream(stream))]
        return PreparedCall(load().tabed_update_weights, args, "tabed_update_weights", args[2])

    def prepare_draft_step(self, rnd, pos, W, H, temperature, u_draft=None, stream=None) -> PreparedCall:
        import torch
        c = self.cfg
        sd = _store_dtype(c)
        vp = C.c_void_p
        args = [C.byref(c), vp(self.ws.data_ptr()), C.c_uint64(rnd), C.c_int32(pos),
                vp(_ptr(W, sd, c.V * c.d, "W")), vp(_ptr(H, sd, c.B * c.n * c.d, "H")),
                vp(self.weights.data_ptr()), vp(_ptr(temperature, torch.float32, c.B, "temperature")),
                vp(_ptr(u_draft, torch.float32, c.B * c.gamma, "u_draft")),
                vp(self.draft_logits.data_ptr()), vp(self.draft_lse.data_ptr()), vp(self.draft_tokens.data_ptr()),
                vp(self.draft_q.data_ptr()), vp(self.draft_flags.data_ptr()), vp(_stream(stream))]
        return PreparedCall(load().tabed_draft_step, args, "tabed_draft_step", args[2])

    def prepare_verify(self, rnd, target_logits, temperature, u_acc=None, u_res=None, stream=None,
                       fused_update=False) -> PreparedCall:
        import torch
        c = self.cfg
        vp = C.c_void_p
        args = [C.byref(c), vp(self.ws.data_ptr()), C.c_uint64(rnd),
                vp(_ptr(target_logits, torch.float32, c.B * (c.gamma + 1) * c.V, "target_logits")),
                vp(self.draft_logits.data_ptr()), vp(self.draft_lse.data_ptr()), vp(self.draft_tokens.data_ptr()),
                vp(self.draft_q.data_ptr()), vp(self.weights.data_ptr()),
                vp(_ptr(temperature, torch.float32, c.B, "temperature")),
                vp(_ptr(u_acc, torch.float32, c.B * c.gamma, "u_acc")), vp(_ptr(u_res, torch.float32, c.B, "u_res")),
                vp(self.accept_len.data_ptr()), vp(self.out_tokens.data_ptr()), vp(self.dev.data_ptr()),
                vp(self.n_valid.data_ptr()), vp(self.verify_flags.data_ptr()),
                vp(self.ring.data_ptr() if fused_update else None), vp(self.ring_head.data_ptr() if fused_update else None),
                vp(self.ring_count.data_ptr() if fused_update else None),
                vp(self.weights.data_ptr() if fused_update else None), vp(_stream(stream))]
        return PreparedCall(load().tabed_verify, args, "tabed_verify", args[2])

    def update_weights(self, first: bool, rnd=0, stream=None):
        tabed_update_weights(self.cfg, self.ws, rnd, None if first else self.dev, None if first else self.n_valid,
                             self.ring, self.ring_head, self.ring_count, self.weights, stream)

    def draft_step(self, rnd, pos, W, H, temperature, u_draft=None, stream=None):
        tabed_draft_step(self.cfg, self.ws, rnd, pos, W, H, self.weights, temperature, self.draft_logits,
                         self.draft_lse, self.draft_tokens, self.draft_q, self.draft_flags, u_draft, stream)

    def verify(self, rnd, target_logits, temperature, u_acc=None, u_res=None, stream=None, fused_update=False):
        """fused_update: the call also opens the next round (window push + next weights, in place)."""
        w = dict(ring=self.ring, ring_head=self.ring_head, ring_count=self.ring_count,
                 next_weights=self.weights) if fused_update else {}
        tabed_verify(self.cfg, self.ws, rnd, target_logits, self.draft_logits, self.draft_lse, self.draft_tokens,
                     self.draft_q, self.weights, temperature, self.accept_len, self.out_tokens, self.dev,
                     self.n_valid, self.verify_flags, u_acc, u_res, stream=stream, **w)
