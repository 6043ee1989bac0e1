"""dsmoe_dispatch_static (the dispatch for callers that cannot allocate: its scratch is a device array inside
the library) against dsmoe_dispatch, through the C ABI: every routing object bit-exact, on two calls in a row,
the second with a smaller input; the context of the static calls has no workspace at all."""
import sys

import numpy as np
import pytest

import dsmoe_inputs as gen
from oracle import dsmoe_oracle as orc

pytestmark = pytest.mark.gpu

KEYS = ("expert_off", "row_token", "row_weight", "tok_off", "tok_rows")


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def routing(torch, cfg, variant):
    inp = gen.make_layer(cfg, variant)
    S = orc.route(inp.x, inp.w_r, inp.b_r).astype(np.float32)
    M = orc.select(S, cfg.mode, cfg.k, np.float32(cfg.eps))
    bits = (M.astype(np.uint64) << np.arange(cfg.E, dtype=np.uint64)[None, :]).sum(axis=1, dtype=np.uint64)
    x = torch.from_numpy(inp.x).cuda().to(torch.bfloat16)
    return x, torch.from_numpy(S).cuda(), torch.from_numpy(bits.view(np.int64)).cuda(), orc.dispatch(M, S)


def compare(torch, r_static, r_plain, r_ref, x, materialize):
    torch.cuda.synchronize()
    nnz = int(r_plain["nnz"][0].item())
    assert nnz == int(r_static["nnz"][0].item()) == r_ref.nnz
    for k in KEYS:
        n = nnz if k in ("row_token", "row_weight", "tok_rows") else r_plain[k].numel()
        assert torch.equal(r_static[k][:n], r_plain[k][:n]), k
    np.testing.assert_array_equal(r_static["expert_off"].cpu().numpy(), r_ref.expert_off)
    np.testing.assert_array_equal(r_static["row_token"].cpu().numpy()[:nnz], r_ref.row_token)
    np.testing.assert_array_equal(r_static["tok_rows"].cpu().numpy()[:nnz], r_ref.tok_rows)
    np.testing.assert_array_equal(r_static["row_weight"].cpu().numpy()[:nnz], r_ref.row_weight)
    if materialize:
        assert torch.equal(r_static["x_perm"][:nnz], r_plain["x_perm"][:nnz])
        assert torch.equal(r_static["x_perm"][:nnz], x[r_static["row_token"][:nnz].long()])


def test_static_dispatch_matches_dispatch_on_two_calls_in_a_row():
    import torch
    import paper_2404_05567_amd as dsmoe
    dsmoe.load_library()
    E, d = 32, 256
    big = gen.LayerConfig("na_big", 41, T=3000, d=d, E=E, f=64, dtype="bf16", mode="threshold", eps=0.02,
                          router_std=1.5 / np.sqrt(d))
    small = big.with_(name="na_small", T=300, mode="topk", k=3)
    plain = dsmoe.Layer(d, 64, E, "bf16", max_tokens=big.T)
    static = dsmoe.Layer(d, 64, E, "bf16", max_tokens=big.T, workspace=False)    # no workspace: nothing lent
    assert static.workspace is None
    bufs = None
    for cfg, materialize in ((big, True), (small, True)):
        say(f"[case] dsmoe_dispatch_static T={cfg.T} E={E} mode={cfg.mode}")
        x, S, bits, r_ref = routing(torch, cfg, 0)
        r_plain = plain.dispatch(x, S, bits, materialize=materialize)
        assert plain.poll_error() == dsmoe.OK
        if bufs is None:
            bufs = static.dispatch(x, S, bits, materialize=materialize, static=True)
        else:
            # the second, smaller call writes into the first call's buffers: what lies past its nnz rows is the
            # first call's and must not matter
            bufs = static.dispatch(x, S, bits, materialize=materialize, static=True, out=bufs)
        assert static.poll_error() == dsmoe.OK
        compare(torch, bufs, r_plain, r_ref, x, materialize)
    # the first size again: what the smaller call left in the array does not leak into a later call
    x, S, bits, r_ref = routing(torch, big, 0)
    r_plain = plain.dispatch(x, S, bits, materialize=False)
    bufs["x_perm"] = None
    bufs = static.dispatch(x, S, bits, static=True, out=bufs)
    compare(torch, bufs, r_plain, r_ref, x, False)


def test_static_dispatch_limits_and_overflow():
    import torch
    import paper_2404_05567_amd as dsmoe
    lib = dsmoe.load_library()
    E, d = 8, 64
    cfg = gen.LayerConfig("na_ovf", 42, T=200, d=d, E=E, f=64, dtype="bf16", mode="topk", k=2, router_std=0.1)
    x, S, bits, r_ref = routing(torch, cfg, 0)
    layer = dsmoe.Layer(d, 64, E, "bf16", max_tokens=cfg.T, max_rows=300, workspace=False)    # needs 400 rows
    r = layer.dispatch(x, S, bits, static=True)
    assert layer.poll_error() == dsmoe.ERR_CAPACITY
    assert layer.poll_error() == dsmoe.OK
    torch.cuda.synchronize()
    assert int(r["expert_off"].abs().sum().item()) == 0 and int(r["nnz"][0].item()) == 0
    # more tokens than the array serves: refused on the host, nothing enqueued
    huge = dsmoe.Layer(d, 64, E, "bf16", max_tokens=1 << 17, max_rows=16, workspace=False)
    from ctypes import c_void_p
    fake = c_void_p(0x1000)
    rc = lib.dsmoe_dispatch_static(huge.ctx, fake, fake, fake, (1 << 16) + 1, fake, fake, fake, fake, fake, fake,
                                   None, None)
    assert rc == dsmoe.ERR_UNSUPPORTED
    assert b"DSMOE_STATIC_DISPATCH_MAX_TOKENS" in lib.dsmoe_last_error(huge.ctx)
