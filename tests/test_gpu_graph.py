"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a caller may capture its calls in a HIP graph.  These tests capture the
one-call and the two-call logits path and the lm_head forward + backward after a warm-up call, replay the graphs
several times with eager work and synchronisations in between, and require every replay to be
bitwise equal to the eager result."""
import sys

import pytest
import torch

import paper_2507_19766_amd as ulorl
import ulorl_inputs as ui

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def _eager_noise():
    # unrelated eager work between replays (allocations, a reduction, a sync)
    x = torch.randn(1 << 20, device=DEV)
    s = float(x.sum())
    torch.cuda.synchronize()
    return s


def test_one_call_path_replays_bitwise_from_a_graph():
    w = ui.shrink(ui.config(2), [700, 300, 1, 523], V=151936 // 8, name="graph_logits")
    say("graph: %s N=%d V=%d" % (w.name, w.N, w.V))
    d = ui.generate(w, DEV)
    p = ulorl.Params(gate_mode=ulorl.GATE_PER_RESPONSE, sigma=7.0, seg_len=w.seg_len)
    ws = torch.empty(ulorl.token_loss_workspace_bytes(w.N, w.V, w.R), dtype=torch.uint8, device=DEV)
    args = (d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    ref, dz_ref = ulorl.token_loss_fwd_bwd(*args, grad_out=1.0, workspace=ws)      # eager; also the warm-up
    torch.cuda.synchronize()
    dz = torch.empty_like(d["logits"])
    out, _ = ulorl.token_loss_fwd_bwd(*args, grad_out=1.0, dlogits=dz, workspace=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ulorl.token_loss_fwd_bwd(*args, grad_out=1.0, dlogits=dz, out=out, workspace=ws)
    for replay in range(3):
        dz.fill_(float("nan"))
        out.loss.fill_(float("nan"))
        out.gcoef.fill_(float("nan"))
        out.mpt_mask.fill_(7)
        _eager_noise()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.loss, ref.loss), replay
        assert torch.equal(out.gcoef, ref.gcoef), replay
        assert torch.equal(out.mpt_mask, ref.mpt_mask), replay
        assert torch.equal(out.counters, ref.counters), replay
        assert torch.equal(dz.view(torch.int16), dz_ref.view(torch.int16)), replay


def test_two_call_path_replays_bitwise_from_a_graph():
    """Forward (statistics by pieces + merge + O(N) kernels) and backward captured together; the
    replays must also match the one-call path, which carries the same bits."""
    w = ui.shrink(ui.config(2), [700, 300, 1, 523], V=151936 // 8, name="graph_two_calls")
    say("graph: %s N=%d V=%d" % (w.name, w.N, w.V))
    d = ui.generate(w, DEV)
    p = ulorl.Params(gate_mode=ulorl.GATE_ALWAYS, seg_len=w.seg_len)
    ws = torch.empty(ulorl.token_loss_workspace_bytes(w.N, w.V, w.R), dtype=torch.uint8, device=DEV)
    args = (d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    ref = ulorl.token_loss_fwd(*args, workspace=ws)                                # eager; also the warm-up
    dz_ref = ulorl.token_loss_bwd(d["logits"], d["token_ids"], ref.lse, ref.gcoef)
    one, dz_one = ulorl.token_loss_fwd_bwd(*args, grad_out=1.0)
    torch.cuda.synchronize()
    assert torch.equal(dz_one.view(torch.int16), dz_ref.view(torch.int16))
    out = ulorl.token_loss_fwd(*args, workspace=ws)
    dz = torch.empty_like(d["logits"])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ulorl.token_loss_fwd(*args, out=out, workspace=ws)
        ulorl.token_loss_bwd(d["logits"], d["token_ids"], out.lse, out.gcoef, dlogits=dz)
    for replay in range(3):
        dz.fill_(float("nan"))
        out.loss.fill_(float("nan"))
        out.lse.fill_(float("nan"))
        out.gcoef.fill_(float("nan"))
        _eager_noise()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.loss, ref.loss) and torch.equal(out.loss, one.loss), replay
        assert torch.equal(out.lse, ref.lse) and torch.equal(out.gcoef, ref.gcoef), replay
        assert torch.equal(out.counters, ref.counters), replay
        assert torch.equal(dz.view(torch.int16), dz_ref.view(torch.int16)), replay


def test_lmhead_forward_and_backward_replay_bitwise_from_a_graph():
    w = ui.shrink(ui.config(5), [300, 212], V=4096 + 1544, hidden=256, seg_len=128, name="graph_lmhead")
    say("graph: %s N=%d Hd=%d V=%d" % (w.name, w.N, w.hidden, w.V))
    d = ui.generate(w, DEV)
    p = ulorl.Params(gate_mode=ulorl.GATE_ALWAYS, seg_len=w.seg_len)
    chunk = 1024
    ws = torch.empty(ulorl.lmhead_workspace_bytes(w.N, w.hidden, w.V, w.R, chunk), dtype=torch.uint8, device=DEV)
    fargs = (d["hidden"], d["weight"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    ref = ulorl.lmhead_token_loss_fwd(*fargs, vocab_chunk=chunk, workspace=ws)
    dH_ref, dW_ref = ulorl.lmhead_token_loss_bwd(d["hidden"], d["weight"], d["token_ids"], ref.lse, ref.gcoef, 1.0,
                                                 vocab_chunk=chunk, workspace=ws)
    torch.cuda.synchronize()
    out = ulorl.lmhead_token_loss_fwd(*fargs, vocab_chunk=chunk, workspace=ws)
    dH = torch.empty_like(dH_ref)
    dW = torch.empty_like(dW_ref)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ulorl.lmhead_token_loss_fwd(*fargs, vocab_chunk=chunk, out=out, workspace=ws)
        ulorl.lmhead_token_loss_bwd(d["hidden"], d["weight"], d["token_ids"], out.lse, out.gcoef, 1.0,
                                    vocab_chunk=chunk, d_hidden=dH, d_weight=dW, workspace=ws)
    for replay in range(3):
        dH.fill_(float("nan"))
        dW.fill_(float("nan"))
        out.lse.fill_(float("nan"))
        _eager_noise()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.loss, ref.loss), replay
        assert torch.equal(out.lse, ref.lse), replay
        assert torch.equal(dH.view(torch.int16), dH_ref.view(torch.int16)), replay
        assert torch.equal(dW.view(torch.int16), dW_ref.view(torch.int16)), replay
