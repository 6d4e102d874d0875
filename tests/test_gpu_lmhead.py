"""GPU parity of the lm_head variant (logits never materialised) and of its MFMA product."""
import sys

import numpy as np
import pytest
import torch

import paper_2507_19766_amd as ulorl
import ulorl_inputs as ui
from parity import params_for, run_lmhead_parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, file=sys.stderr, flush=True)


@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (130, 70, 72), (257, 300, 2048), (1000, 520, 8), (64, 33, 136)])
def test_gemm_tn_bf16_against_fp64(M, N, K):
    g = torch.Generator(device=DEV).manual_seed(M * 1000 + N)
    a = torch.randn(M, K, generator=g, device=DEV).to(torch.bfloat16)
    b = torch.randn(N, K, generator=g, device=DEV).to(torch.bfloat16)
    c = ulorl.gemm_tn_bf16(a, b)
    ref = a.double() @ b.double().T
    bound = 1e-6 * (a.double().abs() @ b.double().abs().T) + 1e-30
    assert torch.all((c.double() - ref).abs() <= bound), float(((c.double() - ref).abs() / bound).max())
    # strided operands (leading dimension > K)
    big = torch.zeros(M, K + 16, device=DEV, dtype=torch.bfloat16)
    big[:, :K] = a
    c2 = ulorl.gemm_tn_bf16(big[:, :K], b)
    assert torch.equal(c, c2)
    # strided result whose pitch allows 16-byte stores while N itself may end inside a vector:
    # same values, and the columns beyond N stay untouched
    ldc = (N + 3) // 4 * 4 + 4
    wide = torch.full((M, ldc), -7.0, device=DEV, dtype=torch.float32)
    ulorl.gemm_tn_bf16(a, b, out=wide[:, :N])
    assert torch.equal(wide[:, :N], c)
    assert torch.all(wide[:, N:] == -7.0)


@pytest.mark.parametrize("tile,group_m", [(0, 0), (1, 0), (0, 1), (0, 7), (1, 64)])
def test_every_compiled_tile_shape(tile, group_m):
    """Both tile shapes / both main loops (direct-to-LDS and register-staged) and other walks of the
    tile grid give the same answers."""
    launch = ulorl.Launch(gemm_tile=tile, gemm_group_m=group_m)
    g = torch.Generator(device=DEV).manual_seed(tile)
    for (M, N, K) in ((300, 520, 192), (256, 256, 72), (1300, 700, 128)):     # K = 72 exercises the ragged-K fallback
        a = torch.randn(M, K, generator=g, device=DEV).to(torch.bfloat16)
        b = torch.randn(N, K, generator=g, device=DEV).to(torch.bfloat16)
        c = ulorl.gemm_tn_bf16(a, b, launch=launch)
        ref = a.double() @ b.double().T
        bound = 1e-6 * (a.double().abs() @ b.double().abs().T) + 1e-30
        assert torch.all((c.double() - ref).abs() <= bound)
    w = ui.shrink(ui.config(5), [150, 120], V=1544, hidden=128, seg_len=64, name="lmhead_tile%d" % tile)
    run_lmhead_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS, tau=0.05), chunk=512, launch=launch)


def test_lmhead_small_ragged_chunks():
    w = ui.shrink(ui.config(5), [120, 83], V=2056, hidden=136, seg_len=32, name="lmhead_small")
    d = ui.generate(w, DEV)
    for mode in (ulorl.GATE_ALWAYS, ulorl.GATE_NEVER):
        run_lmhead_parity(w, params_for(w, gate_mode=mode, tau=0.05), chunk=512, data=d)
    run_lmhead_parity(w, params_for(w, gate_mode=ulorl.GATE_PER_RESPONSE, sigma=100.0, tau=0.05,
                                    is_mode=ulorl.IS_POIS), chunk=8192, data=d, grad_out=-1.5)


def test_lmhead_config5_reduced_rows():
    # the full hidden size and vocabulary of configuration 5, 2 x 512 rows
    w = ui.shrink(ui.config(5), [512, 512], seg_len=256, name="cfg5_reduced")
    res, tt = run_lmhead_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS), chunk=8192, say=say)
    assert tt.n_clip_inactive > 0


def test_lmhead_mpt_mask_fires():
    """A labelled extra case: full hidden size and vocabulary of configuration 5, 2 x 384 rows, a
    third of the hidden rows aligned with one column of W (scaled so that the sampled token's
    probability spreads from ~0.93 to ~1) -- with hidden ~ N(0, 1) . W ~ N(0, 0.02) alone no token
    comes near tau = 0.99 and the mask of Eq. MPTS / I_msk (Sec. 3.2.2) would never be set.
    Mask bit-exact outside |p - tau| < 1e-6, masked tokens carry a zero coefficient and contribute
    exactly nothing to d_hidden (checked in run_lmhead_parity), d_W against the oracle."""
    from dataclasses import replace
    w = replace(ui.shrink(ui.config(5), [384, 384], seg_len=192), align_frac=0.35, name="cfg5_mpt_fires")
    p = params_for(w, gate_mode=ulorl.GATE_ALWAYS)
    res, tt = run_lmhead_parity(w, p, chunk=8192, say=say)
    mask = res.mpt_mask.cpu().numpy().astype(bool)
    assert tt.n_masked >= 20 and int(res.counters[0]) > 0, tt.n_masked
    # some aligned tokens stay below the threshold, and the negative-advantage response is never masked
    prob = np.exp(res.logp.cpu().numpy())
    assert ((prob > 0.9) & (prob < 0.99) & ~mask).sum() >= 5
    assert not mask[384:].any() and mask[:384].any()
    assert bool((res.gcoef[torch.as_tensor(mask, device=DEV)] == 0).all())
    assert bool((res.d_hidden[torch.as_tensor(mask, device=DEV)] == 0).all())
    # the same batch under the per-response gate with sigma between the two responses' mean entropies:
    # only one response's MPTs are masked
    hb = np.sort(tt.resp_entropy)
    if hb[1] - hb[0] > 2e-3:
        sigma = float(0.5 * (hb[0] + hb[1]))
        d = ui.generate(w, DEV)
        r2, tt2 = run_lmhead_parity(w, params_for(w, gate_mode=ulorl.GATE_PER_RESPONSE, sigma=sigma), chunk=8192, data=d)
        assert int(tt2.resp_gate.sum()) == 1


@pytest.mark.parametrize("lengths,V,hidden,chunk", [([300, 212], 4096 + 1544, 256, 1024), ([64], 8192 + 8, 64, 64),
                                                    ([1000, 24], 1544, 128, 2048)])
def test_workspace_is_never_overrun(lengths, V, hidden, chunk):
    """Guard bytes behind the workspace stay untouched by the forward and the backward call (shapes
    with few token tiles and many vocabulary tiles ask for the most vocabulary slices)."""
    w = ui.shrink(ui.config(5), lengths, V=V, hidden=hidden, seg_len=64, name="lmhead_guard")
    d = ui.generate(w, DEV)
    p = ulorl.Params(gate_mode=ulorl.GATE_ALWAYS, seg_len=w.seg_len)
    need = ulorl.lmhead_workspace_bytes(w.N, w.hidden, w.V, w.R, chunk)
    guard = 1 << 20
    buf = torch.full((need + guard,), 0xA5, dtype=torch.uint8, device=DEV)
    ws = buf[:need]
    out = ulorl.lmhead_token_loss_fwd(d["hidden"], d["weight"], d["token_ids"], d["cu_seqlens"], d["advantages"],
                                      d["old_logp"], p, vocab_chunk=chunk, workspace=ws)
    ulorl.lmhead_token_loss_bwd(d["hidden"], d["weight"], d["token_ids"], out.lse, out.gcoef, 1.0, vocab_chunk=chunk,
                                workspace=ws)
    torch.cuda.synchronize()
    assert bool((buf[need:] == 0xA5).all())


def test_lmhead_stats_only_pass():
    """advantages = None: only lse, logp and entropy are produced (how a caller records the
    behaviour policy's log-probs), identical to those of the full forward."""
    w = ui.shrink(ui.config(5), [150, 120], V=1544, hidden=128, seg_len=64, name="lmhead_stats_only")
    d = ui.generate(w, DEV)
    p = ulorl.Params(gate_mode=ulorl.GATE_ALWAYS, seg_len=w.seg_len)
    full = ulorl.lmhead_token_loss_fwd(d["hidden"], d["weight"], d["token_ids"], d["cu_seqlens"], d["advantages"],
                                       d["old_logp"], p, vocab_chunk=512)
    only = ulorl.lmhead_token_loss_fwd(d["hidden"], d["weight"], d["token_ids"], None, None, vocab_chunk=512)
    assert only.loss is None and only.gcoef is None
    for name in ("lse", "logp", "entropy"):
        assert torch.equal(getattr(only, name), getattr(full, name)), name


def _lmhead_bwd_pair(d, w, p, chunk):
    """(forward result, (d_hidden, d_W) over the live rows, the same with every row in the products)"""
    fwd = ulorl.lmhead_token_loss_fwd(d["hidden"], d["weight"], d["token_ids"], d["cu_seqlens"], d["advantages"],
                                      d["old_logp"], p, vocab_chunk=chunk)
    live = ulorl.lmhead_token_loss_bwd(d["hidden"], d["weight"], d["token_ids"], fwd.lse, fwd.gcoef, 1.0, vocab_chunk=chunk)
    dense = ulorl.lmhead_token_loss_bwd(d["hidden"], d["weight"], d["token_ids"], fwd.lse, fwd.gcoef, 1.0, vocab_chunk=chunk,
                                        launch=ulorl.Launch(dense_rows=True))
    torch.cuda.synchronize()
    return fwd, live, dense


def _assert_dw_same_up_to_rounding(a, b):
    a, b = a.float(), b.float()
    # different grouping of the same fp32 terms, then one rounding to bf16: at most an ulp of the larger entries
    assert float((a - b).abs().max()) <= 2.0 ** -7 * float(torch.maximum(a.abs(), b.abs()).max())
    assert float((a - b).abs().mean()) <= 2.0 ** -9 * float(a.abs().mean()) + 1e-30


def test_backward_runs_over_the_live_rows_only():
    """The backward pass gathers the rows with a non-zero coefficient (Sec. 3.2.2: a masked token
    contributes no gradient) and runs its products over those; ULORL_LAUNCH_DENSE_ROWS runs them
    over every row.  Both against the oracle, and against each other: d_hidden bit for bit (a row's
    sums do not depend on which other rows are present), d_W up to the rounding of regrouped sums."""
    from dataclasses import replace
    w = replace(ui.shrink(ui.config(5), [300, 212], V=4096 + 8, hidden=256, seg_len=64), align_frac=0.5,
                name="lmhead_live_rows")
    d = ui.generate(w, DEV)
    p = params_for(w, gate_mode=ulorl.GATE_ALWAYS)
    res, tt = run_lmhead_parity(w, p, chunk=1024, data=d)
    res2, _ = run_lmhead_parity(w, p, chunk=1024, data=d, launch=ulorl.Launch(dense_rows=True))
    dead = int((res.gcoef == 0).sum())
    say("live rows: %d of %d" % (w.N - dead, w.N))
    assert 20 <= dead < w.N - 20
    assert torch.equal(res.d_hidden, res2.d_hidden)
    _assert_dw_same_up_to_rounding(res.d_weight, res2.d_weight)


@pytest.mark.parametrize("n_live", [0, 1, 65])
def test_backward_with_few_or_no_live_rows(n_live):
    """Degenerate live counts: no row at all (every advantage zero: both gradients exactly zero), one
    row, one row more than a 64-column block of the contraction."""
    w = ui.shrink(ui.config(5), [200, 150], V=2056, hidden=128, seg_len=64, name="lmhead_few_live")
    d = ui.generate(w, DEV)
    keep = torch.zeros(w.N, dtype=torch.bool, device=DEV)
    if n_live:
        keep[torch.randperm(w.N, generator=torch.Generator().manual_seed(5))[:n_live].to(DEV)] = True
    d["advantages"] = torch.where(keep, torch.full_like(d["advantages"], 0.75), torch.zeros_like(d["advantages"]))
    p = ulorl.Params(gate_mode=ulorl.GATE_NEVER, seg_len=w.seg_len, eps_low=10.0, eps_high=10.0)
    fwd, (dH, dW), (dH2, dW2) = _lmhead_bwd_pair(d, w, p, chunk=512)
    assert int((fwd.gcoef != 0).sum()) == n_live
    assert torch.equal(dH, dH2)
    assert bool((dH[~keep] == 0).all())
    if n_live == 0:
        assert bool((dH == 0).all()) and bool((dW == 0).all()) and bool((dW2 == 0).all())
    else:
        assert bool((dH[keep].float().abs().sum(dim=1) > 0).all())
        _assert_dw_same_up_to_rounding(dW, dW2)
