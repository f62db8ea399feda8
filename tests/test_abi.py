"""CPU-side checks of the boundary: the library loads, exports every symbol the public header declares,
and rejects bad arguments on the host before anything is enqueued (no GPU is touched here)."""
import ctypes as C
import os
import re

import pytest

from paper_2601_20357_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tabed.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2601_20357_amd import build
        build.build_library()
    return binding.load()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(tabed_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_calls():
    names = declared_functions()
    for must in ("tabed_draft_step", "tabed_update_weights", "tabed_verify", "tabed_workspace_bytes"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in include/tabed.h but not exported by libtabed.so"
    assert sorted(binding.EXPORTS) == declared_functions()


def test_cfg_struct_matches_header_field_order():
    text = open(HEADER).read()
    body = re.search(r"typedef struct tabed_cfg \{(.*?)\} tabed_cfg;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:int32_t|float|uint64_t)\s+([A-Za-z_]+);", body)
    assert fields == [f[0] for f in binding.TabedCfg._fields_]
    assert C.sizeof(binding.TabedCfg) == 9 * 4 + 2 * 4 + 4 + 8      # 4 bytes of padding before the 64-bit seed


def good_cfg(**kw):
    base = dict(V=32000, d=768, n=4, B=16, gamma=5, h=8, w_dtype=1)
    base.update(kw)
    return binding.make_cfg(**base)


def test_workspace_bytes_and_cfg_validation(lib):
    assert binding.tabed_workspace_bytes(good_cfg()) > 2 * 64 * 1000 * 4
    assert binding.tabed_workspace_bytes(good_cfg(V=1, d=8, n=1, B=1, gamma=1, h=1)) > 0
    for bad in (dict(V=0), dict(n=0), dict(n=17), dict(gamma=0), dict(gamma=33), dict(h=-1), dict(B=0),
                dict(d=100), dict(w_dtype=2), dict(tau_w=0.0), dict(eps=0.0), dict(policy=4), dict(distance=3),
                dict(policy=2)):                      # the grid policy is defined for two drafts only
        assert binding.tabed_workspace_bytes(good_cfg(**bad)) == 0, bad
    assert binding.tabed_workspace_bytes(good_cfg(d=100, w_dtype=0)) > 0      # fp32 storage has no d % 8 rule
    assert binding.tabed_workspace_bytes(good_cfg(V=32001)) > 0               # ragged vocabularies are fine
    assert binding.tabed_workspace_bytes(good_cfg(V=262144)) > 0 and binding.tabed_workspace_bytes(good_cfg(V=262145)) == 0
    assert binding.tabed_dev_width(good_cfg()) == 4 and binding.tabed_dev_width(good_cfg(distance=1)) == 4
    assert binding.tabed_dev_width(good_cfg(n=2, policy=2)) == 11 and binding.tabed_dev_width(good_cfg(n=3, policy=2)) == 0


def test_error_codes_are_returned_before_any_launch(lib):
    cfg = good_cfg()
    fake = C.c_void_p(0x1000)          # 16-byte aligned, never dereferenced on the host
    odd = C.c_void_p(0x1008)
    # NULL pointers
    rc = lib.tabed_draft_step(C.byref(cfg), None, 0, 0, *([fake] * 10), None)
    assert rc == -1
    rc = lib.tabed_verify(C.byref(cfg), fake, 0, None, *([fake] * 14), None, None, None, None, None)
    assert rc == -1
    ok15 = [fake] * 7 + [None, None] + [fake] * 5           # u_acc / u_res may be NULL
    rc = lib.tabed_verify(C.byref(cfg), fake, 0, fake, *ok15[1:], fake, None, None, None, None)
    assert rc == -1                     # fused window update: all four pointers or none
    rc = lib.tabed_update_weights(C.byref(cfg), fake, 0, fake, None, fake, fake, fake, fake, None)
    assert rc == -1                     # dev without n_valid
    # position outside the block
    args = [fake] * 4 + [None] + [fake] * 5
    assert lib.tabed_draft_step(C.byref(cfg), fake, 0, 5, *args, None) == -3
    assert lib.tabed_draft_step(C.byref(cfg), fake, 0, -1, *args, None) == -3
    # misaligned base pointer
    args = [odd] + [fake] * 3 + [None] + [fake] * 5
    assert lib.tabed_draft_step(C.byref(cfg), fake, 0, 0, *args, None) == -4
    # invalid / unsupported configuration
    assert lib.tabed_draft_step(C.byref(good_cfg(n=99)), fake, 0, 0, *([fake] * 10), None) == -3
    assert lib.tabed_draft_step(C.byref(good_cfg(V=-4)), fake, 0, 0, *([fake] * 10), None) == -2
    assert lib.tabed_verify(C.byref(good_cfg(policy=2)), fake, 0, *([fake] * 15), None, None, None, None, None) == -2   # needs n = 2
    assert lib.tabed_workspace_init(C.byref(cfg), None, None) == -1
    for code in (0, -1, -2, -3, -4, -5, -6):
        assert lib.tabed_strerror(code).decode() not in ("", "unknown error code")
    assert lib.tabed_strerror(-99).decode() == "unknown error code"
    assert [binding.tabed_kernel_name(i) for i in range(binding.K_COUNT)] == ["lmhead", "sample", "stats", "resid", "weights", "dist", "tree", "body", "null"]


def test_binding_refuses_host_tensors(lib):
    import torch
    cfg = good_cfg(V=8, d=8, n=1, B=1, gamma=1, h=1, w_dtype=0)
    with pytest.raises(binding.TabedError):
        binding.tabed_philox_uniforms(cfg, 0, torch.zeros(4))


def test_tree_and_static_entry_points_validate_before_any_launch(lib):
    cfg = good_cfg()
    fake, odd = C.c_void_p(0x1000), C.c_void_p(0x1008)
    # siblings: width range, position range, a chain needs nothing, NULL and alignment
    sib = lambda width, pos, *ptrs: lib.tabed_draft_siblings(C.byref(cfg), ptrs[0], 0, pos, width, *ptrs[1:], None)
    nine = [fake] * 9
    assert sib(0, 0, fake, *nine[1:]) == -3 and sib(4, 0, fake, *nine[1:]) == -3
    assert sib(2, 5, fake, *nine[1:]) == -3
    assert sib(1, 0, None, *([None] * 8)) == 0                     # tree_width 1: nothing to draw, nothing dereferenced
    assert sib(2, 0, None, *nine[1:]) == -1
    assert sib(2, 0, fake, odd, *nine[2:]) == -4
    # tree verification: hard labels unsupported, leaves required from width 2 on, next_weights must not alias
    args = [fake] * 25
    call = lambda c, width, a: lib.tabed_verify_tree(C.byref(c), fake, 0, width, *a, None)
    assert call(good_cfg(distance=2), 2, args) == -5
    assert call(cfg, 0, args) == -3 and call(cfg, 4, args) == -3
    no_leaf = list(args); no_leaf[1] = None
    assert call(cfg, 2, no_leaf) == -1
    alias = list(args); alias[24] = alias[8]                        # next_weights == weights
    assert call(cfg, 2, alias) == -2
    three_of_four = list(args); three_of_four[21] = None            # ring missing, the rest given
    assert call(cfg, 2, three_of_four) == -1
    # the entry point without a workspace: refuses what does not fit its built-in scratch, before touching the GPU
    big = good_cfg(V=128256, d=2048, n=8, B=64, gamma=5, h=16)
    assert binding.tabed_workspace_bytes(big) > binding.STATIC_SCRATCH_BYTES
    assert lib.tabed_draft_step_static(C.byref(big), 0, 0, *([fake] * 10), None) == binding.ETOOBIG
    assert lib.tabed_draft_step_static(C.byref(cfg), 0, 9, *([fake] * 10), None) == -3
    assert lib.tabed_draft_step_static(C.byref(cfg), 0, 0, None, *([fake] * 9), None) == -1
    assert lib.tabed_strerror(binding.ETOOBIG).decode() not in ("", "unknown error code")


def test_body_entry_points_validate_before_any_launch(lib):
    bc = binding.make_body_cfg(layers=2, d=768, heads=12, d_ff=3072, V=32000, max_ctx=1024)
    assert binding.tabed_body_workspace_bytes(bc, 64) > 64 * 768 * 4
    for bad in (dict(layers=0), dict(layers=17), dict(d=772), dict(d=8200, heads=64), dict(heads=5), dict(heads=192),
                dict(d_ff=3075), dict(V=0), dict(max_ctx=0), dict(max_ctx=9000), dict(rope_theta=-1.0), dict(rms_eps=0.0)):
        kw = dict(layers=2, d=768, heads=12, d_ff=3072, V=32000, max_ctx=1024)
        kw.update(bad)
        assert binding.tabed_body_workspace_bytes(binding.make_body_cfg(**kw), 64) == 0, bad
    assert binding.tabed_body_workspace_bytes(bc, 0) == 0 and binding.tabed_body_workspace_bytes(bc, 70000) == 0
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    fields = re.findall(r"\b(?:int32_t|float)\s+([A-Za-z_]+);", re.search(r"typedef struct tabed_body_cfg \{(.*?)\}", text, flags=re.S).group(1))
    assert fields == [f[0] for f in binding.TabedBodyCfg._fields_]
    wfields = re.findall(r"\*\s*([A-Za-z_]+)(?:\[TABED_BODY_MAX_LAYERS\])?;",
                         re.search(r"typedef struct tabed_body_weights \{(.*?)\}", text, flags=re.S).group(1))
    assert wfields == [f[0] for f in binding.TabedBodyWeights._fields_]
    assert int(re.search(r"#define TABED_BODY_MAX_LAYERS (\d+)", text).group(1)) == binding.BODY_MAX_LAYERS
    fake, odd = 0x1000, 0x1008
    w = binding.TabedBodyWeights()
    w.embed, w.g_final = fake, fake
    for name in ("g_attn", "wqkv", "wo", "g_mlp", "wgu", "wdown"):
        for l in range(2):
            getattr(w, name)[l] = fake
    vp = C.c_void_p
    step = lambda weights, *p: lib.tabed_draft_body_step(C.byref(bc), C.byref(weights), p[0], 64, p[1], 1, 4, *p[2:], None)
    ok = [vp(fake)] * 6                                            # ws, token_src, ctx_len, kcache, vcache, H
    assert lib.tabed_draft_body_step(C.byref(bc), None, ok[0], 64, ok[1], 1, 4, *ok[2:], None) == -1
    assert step(w, None, *ok[1:]) == -1
    assert step(w, vp(odd), *ok[1:]) == -4
    assert lib.tabed_draft_body_step(C.byref(bc), C.byref(w), ok[0], 64, ok[1], 1, 0, *ok[2:], None) == -3    # rows_per_token
    w.wo[1] = None
    assert step(w, *ok) == -1
    w.wo[1] = odd
    assert step(w, *ok) == -4
    assert lib.tabed_draft_body_rollback(64, 4, 5, None, vp(fake), vp(fake), None) == -1
    assert lib.tabed_draft_body_rollback(64, 0, 5, vp(fake), vp(fake), vp(fake), None) == -3
    assert lib.tabed_body_workspace_init(C.byref(bc), 64, None, None) == -1
