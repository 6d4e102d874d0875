"""The torch.autograd entry points hand out exactly what the library calls they forward to produce."""
import pytest
import torch

import paper_2507_19766_amd as ulorl
import ulorl_inputs as ui
from parity import params_for

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)


def test_token_loss_two_call_honours_the_upstream_gradient():
    w = ui.shrink(ui.config(2), [150, 90], V=4096 + 264, seg_len=64, name="autograd_two_call")
    d = ui.generate(w, DEV)
    p = params_for(w, gate_mode=ulorl.GATE_ALWAYS, tau=0.05)
    ref = ulorl.token_loss_fwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    ref_d = ulorl.token_loss_bwd(d["logits"], d["token_ids"], ref.lse, ref.gcoef, grad_out=0.5)
    logits = d["logits"].clone().requires_grad_(True)
    got = []
    loss = ulorl.autograd.token_loss(logits, d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p, results=got)
    assert loss.shape == () and loss.requires_grad
    assert torch.equal(loss.detach().reshape(1), ref.loss)
    (loss * 0.5).backward()
    assert torch.equal(_bits(logits.grad), _bits(ref_d))
    assert torch.equal(got[0].mpt_mask, ref.mpt_mask) and int(got[0].counters[3]) == 0


def test_token_loss_fused_hands_out_the_one_call_gradient():
    w = ui.shrink(ui.config(2), [150, 90], V=4096 + 264, seg_len=64, name="autograd_fused")
    d = ui.generate(w, DEV)
    p = params_for(w, gate_mode=ulorl.GATE_ALWAYS, tau=0.05)
    ref, ref_d = ulorl.token_loss_fwd_bwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    logits = d["logits"].clone().requires_grad_(True)
    loss = ulorl.autograd.token_loss(logits, d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p, fused=True)
    loss.backward()
    assert torch.equal(loss.detach().reshape(1), ref.loss)
    assert torch.equal(_bits(logits.grad), _bits(ref_d))
    # the gradient was formed for an upstream 1: anything else is refused, not silently mis-scaled
    logits2 = d["logits"].clone().requires_grad_(True)
    loss2 = ulorl.autograd.token_loss(logits2, d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p, fused=True)
    with pytest.raises(RuntimeError, match="upstream"):
        (loss2 * 2.0).backward()
    with pytest.raises(ValueError, match="in_place"):
        ulorl.autograd.token_loss(logits2, d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p, in_place=True)


def test_lmhead_token_loss_gradients_to_hidden_and_weight():
    w = ui.shrink(ui.config(5), [120, 83], V=2056, hidden=136, seg_len=32, name="autograd_lmhead")
    d = ui.generate(w, DEV)
    p = params_for(w, gate_mode=ulorl.GATE_ALWAYS, tau=0.05)
    ref = ulorl.lmhead_token_loss_fwd(d["hidden"], d["weight"], d["token_ids"], d["cu_seqlens"], d["advantages"],
                                      d["old_logp"], p, vocab_chunk=512)
    rH, rW = ulorl.lmhead_token_loss_bwd(d["hidden"], d["weight"], d["token_ids"], ref.lse, ref.gcoef, grad_out=-1.5,
                                         vocab_chunk=512)
    hidden = d["hidden"].clone().requires_grad_(True)
    weight = d["weight"].clone().requires_grad_(True)
    loss = ulorl.autograd.lmhead_token_loss(hidden, weight, d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"],
                                            p, vocab_chunk=512)
    (loss * -1.5).backward()
    assert torch.equal(loss.detach().reshape(1), ref.loss)
    assert torch.equal(_bits(hidden.grad), _bits(rH)) and torch.equal(_bits(weight.grad), _bits(rW))
