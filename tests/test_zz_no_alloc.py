"""The entry point that allocates nothing (ulorl_token_loss_fwd_bwd_static: scratch memory in a
static device array) against the workspace entry point it is a variant of: same bits in every
output and in dlogits, on two calls in a row, the second with a smaller input (the array keeps the
first call's contents), and a third in place."""
import pytest
import torch

import paper_2507_19766_amd as ulorl
import ulorl_inputs as ui
from parity import _bits, assert_same_results, params_for

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(w, p, inplace=False):
    d = ui.generate(w, DEV)
    old = None if p.is_mode == ulorl.IS_POIS else d["old_logp"]
    ref, dz_ref = ulorl.token_loss_fwd_bwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], old, p,
                                           grad_out=0.75)
    z = d["logits"].clone() if inplace else d["logits"]
    got, dz = ulorl.token_loss_fwd_bwd_static(z, d["token_ids"], d["cu_seqlens"], d["advantages"], old, p,
                                              grad_out=0.75, inplace=inplace)
    torch.cuda.synchronize()
    assert_same_results(ref, got, "static scratch vs workspace (%s)" % w.name)
    assert torch.equal(_bits(dz), _bits(dz_ref)), "dlogits differ (%s)" % w.name
    assert int(got.counters[3].item()) == 0
    return got


def test_static_scratch_entry_point_matches_the_workspace_one():
    ulorl.init()
    assert ulorl.static_scratch_bytes() == 32 << 20
    # several pieces per row (row-cooperative kernel), two gated responses: the deferred-row pass runs too
    big = ui.shrink(ui.config(2), [700, 300, 420], V=151936 // 2, seg_len=256, name="static_big")
    r1 = _both(big, params_for(big, gate_mode=ulorl.GATE_PER_RESPONSE, sigma=100.0))
    assert int(r1.counters[0].item()) >= 0
    # a smaller input right after: fewer rows, fewer pieces per row, other gate
    small = ui.shrink(ui.config(2), [90, 37], V=5000, seg_len=16, name="static_small")
    _both(small, params_for(small, gate_mode=ulorl.GATE_ALWAYS, tau=0.5))
    # fp32 storage, in place
    f32w = ui.shrink(ui.config(1), [33, 64], V=4100, seg_len=8, name="static_f32")
    _both(f32w, params_for(f32w, gate_mode=ulorl.GATE_NEVER), inplace=True)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    # 2^20 rows of 151936 bf16 logits would need 80 MB of exchange slots: refused on the host, before
    # any pointer is touched (the fake pointers below are never dereferenced)
    import ctypes
    lib = ulorl.load_library()
    vp = ctypes.c_void_p
    cp = ulorl.Params().to_c()
    rc = lib.ulorl_token_loss_fwd_bwd_static(
        vp(0x1000), 1, 1 << 20, 151936, 151936, vp(0x2000), vp(0x3000), 1, None, vp(0x4000), vp(0x5000),
        ctypes.byref(cp), 1.0, vp(0x6000), vp(0x7000), vp(0x8000), vp(0x9000), vp(0xa000), None, None, None, None,
        None, None, None, vp(0x20000), None, None)
    assert rc == -8
    assert "static" in ulorl.status_string(-8)


def test_static_scratch_entry_point_replays_from_a_graph():
    """What the entry point is for: a caller under HIP graph capture, where nothing may be allocated.
    After ulorl_init() and a warm-up call the static-scratch call is captured, replayed three times
    with eager work in between (another static call on a different input among it: the scratch array is
    shared and keeps that call's contents), and every replay must carry the bits of the eager result."""
    ulorl.init()
    w = ui.shrink(ui.config(2), [500, 260, 3], V=151936 // 4, seg_len=128, name="static_graph")
    d = ui.generate(w, DEV)
    p = params_for(w, gate_mode=ulorl.GATE_PER_RESPONSE, sigma=100.0, tau=0.5)
    args = (d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    ref, dz_ref = ulorl.token_loss_fwd_bwd(*args)
    dz = torch.empty_like(d["logits"])
    out, _ = ulorl.token_loss_fwd_bwd_static(*args, dlogits=dz)                  # warm-up, allocates the outputs
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ulorl.token_loss_fwd_bwd_static(*args, dlogits=dz, out=out)
    other = ui.shrink(ui.config(2), [90, 37], V=5000, seg_len=16, name="static_graph_other")
    do = ui.generate(other, DEV)
    for replay in range(3):
        dz.fill_(float("nan"))
        out.loss.fill_(float("nan"))
        out.gcoef.fill_(float("nan"))
        # eager work between the replays, on the same scratch array
        ulorl.token_loss_fwd_bwd_static(do["logits"], do["token_ids"], do["cu_seqlens"], do["advantages"], do["old_logp"],
                                        params_for(other, gate_mode=ulorl.GATE_ALWAYS))
        float(torch.randn(1 << 18, device=DEV).sum())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_same_results(ref, out, "graph replay %d of the static-scratch call" % replay)
        assert torch.equal(_bits(dz), _bits(dz_ref)), replay
