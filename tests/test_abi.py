"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments on the
host before touching a device (no GPU needed)."""
import ctypes
import os
import re
from ctypes import byref, c_size_t, c_void_p

import pytest

import paper_2404_05567_amd as dsmoe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dsmoe.LIB_PATH):
        from paper_2404_05567_amd import build
        build.build(verbose=False)
    return dsmoe.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dsmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dsmoe_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(dsmoe.EXPORTS) == names


def make(lib, **kw):
    d = dict(d_model=256, d_ff=64, n_experts=8, dtype=dsmoe.F32, max_tokens=128, max_rows=1024)
    d.update(kw)
    ctx = c_void_p()
    rc = lib.dsmoe_create(byref(dsmoe.Desc(**d)), byref(ctx))
    return rc, ctx


def test_create_validates_the_descriptor(lib):
    rc, ctx = make(lib)
    assert rc == dsmoe.OK and ctx.value
    n = c_size_t()
    assert lib.dsmoe_workspace_bytes(ctx, byref(n)) == dsmoe.OK and n.value > 0
    assert lib.dsmoe_destroy(ctx) == dsmoe.OK
    assert make(lib, n_experts=128)[0] == dsmoe.ERR_UNSUPPORTED
    assert make(lib, n_experts=12)[0] == dsmoe.ERR_UNSUPPORTED
    assert make(lib, d_model=250)[0] == dsmoe.ERR_UNSUPPORTED
    assert make(lib, d_ff=40)[0] == dsmoe.ERR_UNSUPPORTED
    assert make(lib, dtype=7)[0] == dsmoe.ERR_UNSUPPORTED
    assert make(lib, d_model=0)[0] == dsmoe.ERR_INVALID_ARG
    assert make(lib, max_rows=128 * 8 + 1)[0] == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_create(None, byref(c_void_p())) == dsmoe.ERR_INVALID_ARG


def test_calls_reject_bad_arguments_before_any_device_work(lib):
    rc, ctx = make(lib)
    assert rc == dsmoe.OK
    fake = c_void_p(0x1000)     # aligned, never dereferenced on these paths
    odd = c_void_p(0x1004)
    s = None
    assert lib.dsmoe_route(ctx, None, fake, None, 4, fake, s) == dsmoe.ERR_INVALID_ARG
    assert b"null pointer" in lib.dsmoe_last_error(ctx)
    assert lib.dsmoe_route(ctx, odd, fake, None, 4, fake, s) == dsmoe.ERR_INVALID_ARG
    assert b"aligned" in lib.dsmoe_last_error(ctx)
    assert lib.dsmoe_route(ctx, fake, fake, None, -1, fake, s) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_route(ctx, fake, fake, None, 129, fake, s) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_TOPK, 0, 0.0, fake, None, s) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_TOPK, 9, 0.0, fake, None, s) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_THRESHOLD, 0, -0.5, fake, None, s) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_THRESHOLD, 0, float("nan"), fake, None, s) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_select(ctx, fake, 4, 5, 1, 0.0, fake, None, s) == dsmoe.ERR_INVALID_ARG
    # the normalised threshold of the paper goes with the threshold modes only, and is validated like eps
    norm = dsmoe.SEL_NORMALISED
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_TOPK | norm, 2, 0.5, fake, None, s) == dsmoe.ERR_INVALID_ARG
    assert b"DSMOE_SEL_NORMALISED" in lib.dsmoe_last_error(ctx)
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_THRESHOLD | norm, 0, -0.5, fake, None, s) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_THRESHOLD | norm, 0, float("inf"), fake, None, s) \
        == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_select(ctx, fake, 0, dsmoe.SEL_THRESHOLD | norm, 0, 0.48, fake, None, s) == dsmoe.OK   # T = 0
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_THRESHOLD_TOPK | norm, 0, 0.48, fake, None, s) == dsmoe.ERR_WORKSPACE
    assert lib.dsmoe_sparse_fwd(ctx, fake, fake, None, fake, fake, fake, 4, 7 | norm, 2, 0.1, fake, s) \
        == dsmoe.ERR_WORKSPACE      # the workspace check comes first ...
    # calls that need the workspace refuse to run without one
    assert lib.dsmoe_sparse_fwd(ctx, fake, fake, None, fake, fake, fake, 4, dsmoe.SEL_TOPK, 2, 0.0, fake, s) \
        == dsmoe.ERR_WORKSPACE
    assert lib.dsmoe_expert_ffn(ctx, fake, None, fake, fake, fake, fake, fake, fake, s) == dsmoe.ERR_WORKSPACE
    # the later entry points: Threshold-TopK needs the workspace, the loss needs tokens, the expert kind is checked
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_THRESHOLD_TOPK, 0, 0.1, fake, None, s) == dsmoe.ERR_WORKSPACE
    assert lib.dsmoe_select(ctx, fake, 4, dsmoe.SEL_THRESHOLD_TOPK, 0, -1.0, fake, None, s) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_mi_loss(ctx, fake, 4, fake, fake, s) == dsmoe.ERR_WORKSPACE
    assert lib.dsmoe_set_expert_kind(ctx, 7) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_set_expert_kind(ctx, dsmoe.EXPERT_GELU) == dsmoe.OK
    assert lib.dsmoe_set_expert_kind(ctx, dsmoe.EXPERT_SWIGLU) == dsmoe.OK
    import ctypes as ct
    bad_alpha = ct.c_float(float("inf"))
    assert lib.dsmoe_dense_bwd_mi(ctx, fake, fake, fake, fake, fake, fake, fake, 4, fake, fake, fake, None, fake, fake,
                                  fake, bad_alpha, s) == dsmoe.ERR_INVALID_ARG
    # the dispatch that needs no workspace: arguments and its size limit are checked before any device work
    st = lambda **kw: lib.dsmoe_dispatch_static(ctx, fake, kw.get("probs", fake), fake, kw.get("T", 4), fake, fake, fake,
                                                kw.get("tok_off", fake), fake, fake, None, s)
    assert st(T=-1) == dsmoe.ERR_INVALID_ARG
    assert st(T=129) == dsmoe.ERR_INVALID_ARG                 # beyond the context's max_tokens
    assert st(probs=None) == dsmoe.ERR_INVALID_ARG
    assert st(tok_off=odd) == dsmoe.ERR_INVALID_ARG
    assert b"dsmoe_dispatch_static" in lib.dsmoe_last_error(ctx)
    rc_big, big = make(lib, max_tokens=1 << 17, max_rows=16)
    assert rc_big == dsmoe.OK
    assert lib.dsmoe_dispatch_static(big, fake, fake, fake, (1 << 16) + 1, fake, fake, fake, fake, fake, fake, None, s) \
        == dsmoe.ERR_UNSUPPORTED
    assert b"DSMOE_STATIC_DISPATCH_MAX_TOKENS" in lib.dsmoe_last_error(big)
    assert lib.dsmoe_destroy(big) == dsmoe.OK
    assert lib.dsmoe_set_workspace(ctx, None, 1 << 20) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_set_workspace(ctx, c_void_p(0x1010), 1 << 30) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_set_workspace(ctx, fake, 16) == dsmoe.ERR_WORKSPACE
    assert lib.dsmoe_destroy(ctx) == dsmoe.OK


def test_attention_layer_entry_points_validate_on_the_host(lib):
    def make_moa(**kw):
        d = dict(d_model=256, n_experts=8, n_head=2, d_head=64, dtype=dsmoe.BF16, max_tokens=64)
        d.update(kw)
        ctx = c_void_p()
        return lib.dsmoe_moa_create(byref(dsmoe.MoaDesc(**d)), byref(ctx)), ctx

    assert make_moa(dtype=dsmoe.F32)[0] == dsmoe.ERR_UNSUPPORTED
    assert make_moa(d_head=96)[0] == dsmoe.ERR_UNSUPPORTED
    assert make_moa(n_experts=12)[0] == dsmoe.ERR_UNSUPPORTED
    assert make_moa(d_model=100)[0] == dsmoe.ERR_UNSUPPORTED
    assert make_moa(n_head=0)[0] == dsmoe.ERR_INVALID_ARG
    rc, ctx = make_moa()
    assert rc == dsmoe.OK and ctx.value
    n = c_size_t()
    assert lib.dsmoe_moa_workspace_bytes(ctx, byref(n)) == dsmoe.OK
    # scores, masks, counts, row index, Q and the weighted attention outputs
    assert n.value >= 64 * 8 * 4 + 64 * 8 + 2 * (8 * 64 * 128 * 2)
    fake, odd, s = c_void_p(0x1000), c_void_p(0x1004), None
    import ctypes as ct
    one = ct.c_float(1.0)
    call = lambda **kw: lib.dsmoe_moa_fwd(
        ctx, kw.get("x", fake), fake, None, fake, fake, fake, fake, kw.get("T", 4), kw.get("L", 8),
        kw.get("mode", dsmoe.SEL_TOPK), kw.get("k", 2), ct.c_float(kw.get("eps", 0.0)), kw.get("scale", one), fake, s)
    assert call() == dsmoe.ERR_WORKSPACE
    assert b"workspace" in lib.dsmoe_moa_last_error(ctx)
    assert call(T=65) == dsmoe.ERR_INVALID_ARG
    assert call(T=4, L=3) == dsmoe.ERR_INVALID_ARG
    assert call(k=0) == dsmoe.ERR_INVALID_ARG
    assert call(mode=dsmoe.SEL_THRESHOLD, eps=-1.0) == dsmoe.ERR_INVALID_ARG
    assert call(mode=dsmoe.SEL_THRESHOLD_TOPK) == dsmoe.ERR_INVALID_ARG
    assert call(scale=ct.c_float(float("nan"))) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_moa_routing(ctx, 4, fake, fake, s) == dsmoe.ERR_WORKSPACE
    assert lib.dsmoe_moa_set_workspace(ctx, c_void_p(0x1010), 1 << 30) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_moa_set_workspace(ctx, fake, 16) == dsmoe.ERR_WORKSPACE
    assert lib.dsmoe_moa_set_workspace(ctx, fake, n.value) == dsmoe.OK      # only recorded, not touched
    assert call(x=None) == dsmoe.ERR_INVALID_ARG
    assert call(x=odd) == dsmoe.ERR_INVALID_ARG
    assert call(T=0) == dsmoe.OK
    # backward: scratch size query, and the call is refused unless the dense forward of the same shape came before
    nb = c_size_t()
    assert lib.dsmoe_moa_bwd_scratch_bytes(ctx, 4, 8, byref(nb)) == dsmoe.OK
    assert nb.value >= 8 * 4 * 2 * 32 * 2       # at least the attention probabilities, key axis padded to 32
    assert lib.dsmoe_moa_bwd_scratch_bytes(ctx, 4, 3, byref(nb)) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_moa_bwd_scratch_bytes(None, 4, 8, byref(nb)) == dsmoe.ERR_INVALID_ARG
    bwd = lambda **kw: lib.dsmoe_moa_bwd(ctx, fake, fake, fake, fake, fake, fake, fake, kw.get("T", 4), kw.get("L", 8),
                                         kw.get("scale", one), fake, fake, fake, None, fake, fake, fake, fake, s)
    assert bwd(T=0) == dsmoe.ERR_INVALID_ARG
    assert bwd(T=65) == dsmoe.ERR_INVALID_ARG
    assert bwd(L=3) == dsmoe.ERR_INVALID_ARG
    assert bwd(scale=ct.c_float(float("inf"))) == dsmoe.ERR_INVALID_ARG
    assert bwd() == dsmoe.ERR_INVALID_ARG and b"dsmoe_moa_fwd" in lib.dsmoe_moa_last_error(ctx)
    assert lib.dsmoe_moa_bwd(None, fake, fake, fake, fake, fake, fake, fake, 4, 8, one, fake, fake, fake, None, fake,
                             fake, fake, fake, s) == dsmoe.ERR_INVALID_ARG
    assert lib.dsmoe_moa_destroy(ctx) == dsmoe.OK
    assert lib.dsmoe_moa_destroy(None) == dsmoe.ERR_INVALID_ARG


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(dsmoe, "_lib", None)
    monkeypatch.setattr(dsmoe, "LIB_PATH", str(tmp_path / "libdsmoe.so"))
    with pytest.raises(ImportError):
        dsmoe.load_library()
