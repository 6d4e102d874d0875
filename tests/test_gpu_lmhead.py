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
