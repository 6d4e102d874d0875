"""Full-size parity on the workload configurations, in the launch configuration the benchmark
times.  Every row's log-softmax statistics and every token's terms are compared with the fp64
oracle (the logits are streamed to the host in blocks); the gradient is compared on sampled
rows, and by properties (exact zero rows) elsewhere."""
import sys

import numpy as np
import pytest
import torch

import paper_2507_19766_amd as ulorl
import ulorl_inputs as ui
from parity import params_for, run_streamed_parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def _generate(w):
    say("generating %s (N=%d, V=%d)" % (w.name, w.N, w.V))
    d = ui.generate(w, DEV)
    torch.cuda.synchronize()
    return d


def test_cfg2_full_size_static_mask_and_mixed_gates():
    w = ui.config(2)
    d = _generate(w)
    res, tt = run_streamed_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS), d, inplace=False, say=say)
    assert tt.n_masked > 50 and tt.n_clip_inactive > 500
    # per-response gate with sigma midway between two responses' mean entropies (oracle values)
    s = np.sort(tt.resp_entropy)
    gaps = np.diff(s)
    j = int(np.argmax(gaps))
    assert gaps[j] > 1e-3
    sigma = 0.5 * (s[j] + s[j + 1])
    p = params_for(w, gate_mode=ulorl.GATE_PER_RESPONSE, sigma=float(sigma))
    old = d["old_logp"]
    r2 = ulorl.token_loss_fwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], old, p)
    expect_gate = (tt.resp_entropy < np.float32(sigma)).astype(np.uint8)
    assert 0 < expect_gate.sum() < w.R
    np.testing.assert_array_equal(r2.resp_gate.cpu().numpy(), expect_gate)
    resp = np.repeat(np.arange(w.R), w.lengths)
    np.testing.assert_array_equal(r2.mpt_mask.cpu().numpy(), tt.mask * expect_gate[resp])


def test_cfg3_full_size_varlen_in_place():
    w = ui.config(3)
    d = _generate(w)
    res, tt = run_streamed_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS), d, inplace=True, say=say)
    seg = res.segment_out.cpu().numpy()
    assert seg.max() == (max(w.lengths) - 1) // w.seg_len
    assert tt.n_masked > 50


def test_cfg4_full_size_ultra_long_in_place():
    w = ui.config(4)
    d = _generate(w)
    res, tt = run_streamed_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS), d, inplace=True, say=say)
    assert tt.n_masked > 200 and tt.n_pos == w.N
    assert int(res.segment_out.max()) == 7


def test_cfg4_full_size_one_call_in_place():
    """The configuration and the call the benchmark times: 131072 x 151936 bf16, one call, in place."""
    w = ui.config(4)
    d = _generate(w)
    res, tt = run_streamed_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS), d, inplace=True, say=say,
                                  one_call=True)
    assert tt.n_masked > 200 and tt.n_pos == w.N
    assert int(res.counters[3].item()) == 0


def test_cfg3_full_size_one_call_with_a_response_gate():
    """Ragged responses, one call, in place, with the per-response entropy gate placed between two
    responses' mean entropies: the members of the MPT set wait for the gate."""
    w = ui.config(3)
    d = _generate(w)
    y = d["token_ids"].cpu().numpy()
    from parity import oracle_row_stats_streamed
    _, _, H, _ = oracle_row_stats_streamed(d["logits"], y)
    cu = w.cu_seqlens
    hbar = np.sort(np.array([H[cu[i]:cu[i + 1]].mean() for i in range(w.R)]))
    gaps = np.diff(hbar)
    j = int(np.argmax(gaps))
    assert gaps[j] > 1e-3
    sigma = float(0.5 * (hbar[j] + hbar[j + 1]))
    res, tt = run_streamed_parity(w, params_for(w, gate_mode=ulorl.GATE_PER_RESPONSE, sigma=sigma), d, inplace=True,
                                  say=say, one_call=True)
    assert 0 < int(tt.resp_gate.sum()) < w.R and tt.n_masked > 10


def test_cfg5_full_size_lmhead_variant():
    """Configuration 5 at full size (32768 x 2048 x 151936): the forward outputs and dHidden of
    sampled rows against the oracle (each depends only on its own row once the static gate and
    the denominator are fixed), dW against the unfused GPU path (materialised bf16 logits ->
    token loss -> stock GEMM), which is an agreement check, not a parity claim."""
    import oracle
    from parity import LMHEAD_ATOL, assert_close, f32, oracle_terms, raw_bf16, rtol_for
    w = ui.config(5)
    d = _generate(w)
    p = params_for(w, gate_mode=ulorl.GATE_ALWAYS)
    hidden, weight = d["hidden"], d["weight"]
    res = ulorl.lmhead_token_loss_fwd(hidden, weight, d["token_ids"], d["cu_seqlens"], d["advantages"],
                                      d["old_logp"], p, vocab_chunk=8192)
    dH, dW = ulorl.lmhead_token_loss_bwd(hidden, weight, d["token_ids"], res.lse, res.gcoef, vocab_chunk=8192)
    torch.cuda.synchronize()
    say("gpu forward+backward done")

    rows = np.unique(np.concatenate([[0, w.N - 1], np.random.RandomState(11).choice(w.N, 190, replace=False)]))
    rt = torch.as_tensor(rows, device=DEV)
    hr, wr = raw_bf16(hidden[rt]), raw_bf16(weight)
    z = oracle.lmhead_logits(hr, wr)
    y = d["token_ids"][rt].cpu().numpy()
    o_lse, o_logp, o_H = oracle.row_stats(z, y)
    rtol = rtol_for("bf16")
    assert_close("lse", res.lse[rt].cpu().numpy(), o_lse, rtol, atol=LMHEAD_ATOL)
    assert_close("logp", res.logp[rt].cpu().numpy(), o_logp, rtol, atol=LMHEAD_ATOL)
    assert_close("entropy", res.entropy[rt].cpu().numpy(), o_H, rtol, atol=LMHEAD_ATOL)
    adv = d["advantages"][rt].cpu().numpy()
    old = d["old_logp"][rt].cpu().numpy()
    tt = oracle_terms(o_logp, o_H, [0, len(rows)], adv, old, p, denominator=float(w.N))
    near = (np.abs(np.exp(o_logp) - f32(p.tau)) < 2e-5) | (np.abs(tt.ratio - 0.8) < 2e-5) | (np.abs(tt.ratio - 1.2) < 2e-5)
    np.testing.assert_array_equal(res.mpt_mask[rt].cpu().numpy()[~near], tt.mask[~near])
    assert_close("gcoef", res.gcoef[rt].cpu().numpy()[~near], tt.gcoef[~near], 3e-5, atol=0.0)
    g = tt.gcoef.copy()
    g[near] = res.gcoef[rt].cpu().numpy()[near]
    dz = oracle.dlogits(z, y, o_lse, g)
    wd = oracle.bf16_to_f64(wr)
    ref_dH = dz @ wd.T
    bound = 2.0 ** -8 * (np.abs(dz) @ np.abs(wd).T) + 2.0 ** -8 * np.abs(ref_dH) + 1e-12
    got = dH[rt].float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref_dH) <= bound)
    assert np.abs(got - ref_dH).mean() / np.abs(ref_dH).mean() < 3e-3
    say("sampled rows ok (%d rows, %d near a discontinuity)" % (len(rows), int(near.sum())))
    del z, dz, wd

    # whole-batch properties: loss from the per-token outputs; counters
    assert int(res.counters[3]) == 0 and int(res.counters[2]) == 16384
    # unfused GPU path for dW
    logits = torch.matmul(hidden, weight)                      # materialised, rounded to bf16
    r2 = ulorl.token_loss_fwd(logits, d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    # the loss is a difference of two sums of about 0.5 (advantages +1 / -1): bf16 logits move it by ~1e-5
    assert abs(r2.loss.item() - res.loss.item()) < 1e-4
    # same coefficients on both sides: a token whose ratio sits within the bf16 noise of a clip edge
    # would otherwise flip its whole gradient row on one side only
    ulorl.token_loss_bwd(logits, d["token_ids"], res.lse, res.gcoef, inplace=True)
    dW2 = torch.matmul(hidden.T, logits)                       # [Hd, V]
    a, b = dW.float(), dW2.float()
    rel = float((a - b).norm() / b.norm())
    say("dW fused vs unfused: relative Frobenius error %.3e" % rel)
    assert rel < 2e-3
    dH2 = torch.matmul(logits, weight.T)
    relh = float((dH.float() - dH2.float()).norm() / dH2.float().norm())
    say("dHidden fused vs unfused: relative Frobenius error %.3e" % relh)
    assert relh < 2e-3
