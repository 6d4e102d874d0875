"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs.  Oracle-sized cases compare every element; see test_gpu_fullsize.py for the
full-size configurations."""
import numpy as np
import pytest
import torch

import oracle
import paper_2507_19766_amd as ulorl
import ulorl_inputs as ui
from parity import (assert_close, check_dlogits, f32, oracle_terms, params_for, rtol_for,
                    run_full_parity, sigma_between_responses)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _host(d):
    return ui.to_numpy_logits(d["logits"]), d["token_ids"].cpu().numpy()


# ------------------------------------------------------------------ configuration 1 (fp32, whole)

def test_cfg1_sais_per_response_gate():
    w = ui.config(1)
    d = ui.generate(w, DEV)
    hl, y = _host(d)
    sigma = sigma_between_responses(hl, y, w.cu_seqlens)
    p = params_for(w, sigma=sigma, gate_mode=ulorl.GATE_PER_RESPONSE)
    res, tt, info = run_full_parity(w, p, data=d)
    assert tt.resp_gate.sum() == 1                      # one response gated, one not


def test_cfg1_static_masking_and_paper_sigma():
    w = ui.config(1)
    d = ui.generate(w, DEV)
    res, tt, _ = run_full_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS), data=d)
    assert tt.n_masked > 0
    # with the paper's sigma = 0.2 these high-entropy rows never trigger the gate
    res2, tt2, _ = run_full_parity(w, params_for(w), data=d)
    assert tt2.n_masked == 0 and int(res2.counters[0]) == 0


def test_cfg1_pois_and_global_gate():
    w = ui.config(1)
    d = ui.generate(w, DEV)
    res, tt, _ = run_full_parity(w, params_for(w, is_mode=ulorl.IS_POIS, gate_mode=ulorl.GATE_ALWAYS),
                                 data=d)
    assert torch.all(res.ratio == 1.0) and int(res.counters[1]) == 0
    run_full_parity(w, params_for(w, gate_mode=ulorl.GATE_GLOBAL, sigma=100.0), data=d)
    run_full_parity(w, params_for(w, gate_mode=ulorl.GATE_NEVER, denominator=5000.0), data=d,
                    grad_out=-2.5)


# ------------------------------------------------------------------ bf16, Qwen3-sized vocabulary

def test_cfg2_recipe_small_ragged_responses():
    w = ui.shrink(ui.config(2), [700, 300, 1100, 205], seg_len=256)
    d = ui.generate(w, DEV)
    hl, y = _host(d)
    sigma = sigma_between_responses(hl, y, w.cu_seqlens)
    rows = np.random.RandomState(3).choice(w.N, 48, replace=False)
    p = params_for(w, sigma=sigma)
    res, tt, _ = run_full_parity(w, p, dz_rows=rows, data=d)
    assert 0 < tt.resp_gate.sum() < 4
    res, tt, _ = run_full_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS), dz_rows=rows, data=d)
    assert tt.n_masked > 0 and tt.n_clip_inactive > 0


def test_cfg4_recipe_small_in_place():
    w = ui.shrink(ui.config(4), [1500], seg_len=200)
    d = ui.generate(w, DEV)
    pristine = d["logits"].clone()
    p = params_for(w, gate_mode=ulorl.GATE_ALWAYS)
    rows = np.concatenate([np.arange(8), np.random.RandomState(4).choice(w.N, 40, replace=False)])
    res, tt, info = run_full_parity(w, p, dz_rows=rows, data=d)         # out of place
    dz_out = info["dz"]
    assert torch.equal(d["logits"], pristine)
    dz_in = ulorl.token_loss_bwd(d["logits"], d["token_ids"], res.lse, res.gcoef, inplace=True)
    assert dz_in.data_ptr() == d["logits"].data_ptr()
    assert torch.equal(dz_in.view(torch.int16), dz_out.view(torch.int16))  # bitwise the same
    seg = res.segment_out.cpu().numpy()
    np.testing.assert_array_equal(seg, np.arange(1500) // 200)
    assert np.all(np.abs(tt.ratio[seg == 0] - 1.0) < 1e-5)               # first segment on-policy
    assert np.abs(tt.ratio[seg == 6] - 1.0).max() > 0.05                 # later ones are stale


def test_heavily_masked_batch_takes_the_write_only_path():
    # spike +20: most peaked rows reach p >= 0.99 and are removed (labelled extra case)
    from dataclasses import replace
    w = replace(ui.shrink(ui.config(4), [600], seg_len=100), spike_boost=22.0, name="cfg4_spike22")
    rows = np.arange(0, 600, 7)
    res, tt, _ = run_full_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS), dz_rows=rows)
    assert tt.n_masked > 100


# ------------------------------------------------------------------ ragged shapes and edge cases

@pytest.mark.parametrize("dtype,V", [("f32", 4099), ("f32", 3), ("f32", 4 * 256 * 4 * 2 + 4 * 77 + 1),
                                     ("bf16", 1003), ("bf16", 5), ("bf16", 8 * 256 * 4 * 2 + 8 * 77 + 5),
                                     ("bf16", 8 * 1024 * 8 + 8)])
@pytest.mark.parametrize("per_row", [False, True])
def test_ragged_vocab_and_launch_shapes(dtype, V, per_row):
    """Vocabulary sizes that end inside a vector, inside a piece and inside a loop trip, padded rows
    (stride > V), by the piece-wise kernels and (per_row) by one looping workgroup per row."""
    base = ui.config(1) if dtype == "f32" else ui.config(2)
    w = ui.shrink(base, [9, 1, 23], V=V, seg_len=4, name="ragged_%s_%d" % (dtype, V))
    dev = torch.device(DEV)
    vec = 4 if dtype == "f32" else 8
    stride = (V + vec - 1) // vec * vec + 2 * vec          # padded rows: stride > V
    d = ui.generate(w, DEV)
    buf = torch.full((w.N, stride), float("nan"), dtype=w.torch_dtype(), device=dev)
    buf[:, :V] = d["logits"]
    d["logits"] = buf[:, :V]
    res, tt, info = run_full_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS, tau=0.5), data=d,
                                    same_bits=not per_row, launch=ulorl.Launch(per_row=per_row))
    # in place on the padded buffer: same bits, and the padding columns stay untouched
    dz_out = info["dz"]
    assert dz_out.stride(0) == stride
    dz_in = ulorl.token_loss_bwd(d["logits"], d["token_ids"], res.lse, res.gcoef, inplace=True)
    as_int = torch.int32 if dtype == "f32" else torch.int16
    assert torch.equal(dz_in.contiguous().view(as_int), dz_out.contiguous().view(as_int))
    assert torch.isnan(buf[:, V:]).all()


def test_single_row_single_token_and_empty_response():
    w = ui.shrink(ui.config(1), [1], V=512, seg_len=1, name="one_row")
    run_full_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS))
    # an empty response in the middle of the batch
    w = ui.shrink(ui.config(1), [5, 4], V=256, seg_len=2, name="with_empty")
    d = ui.generate(w, DEV)
    cu = torch.tensor([0, 5, 5, 9], dtype=torch.int32, device=DEV)
    p = params_for(w, gate_mode=ulorl.GATE_PER_RESPONSE, sigma=100.0)
    res = ulorl.token_loss_fwd(d["logits"], d["token_ids"], cu, d["advantages"], d["old_logp"], p)
    hl, y = _host(d)
    o_lse, o_logp, o_H = oracle.row_stats(hl, y)
    tt = oracle_terms(o_logp, o_H, [0, 5, 5, 9], d["advantages"].cpu().numpy(), d["old_logp"].cpu().numpy(), p)
    np.testing.assert_array_equal(res.resp_gate.cpu().numpy(), tt.resp_gate)
    assert list(tt.resp_gate) == [1, 0, 1]
    assert_close("resp_entropy", res.resp_entropy.cpu().numpy(), tt.resp_entropy, 1e-5)
    np.testing.assert_array_equal(res.mpt_mask.cpu().numpy(), tt.mask)
    np.testing.assert_array_equal(res.segment_out.cpu().numpy(), tt.seg)
    assert_close("loss", res.loss.item(), tt.loss, 1e-5, atol=1e-7)


def test_all_masked_and_none_masked():
    V = 1024
    N = 40
    z = torch.zeros(N, V, device=DEV)
    z[:, 17] = 30.0                                       # every row: p(17) ~ 1
    y = torch.full((N,), 17, dtype=torch.int32, device=DEV)
    cu = torch.tensor([0, N], dtype=torch.int32, device=DEV)
    adv = torch.ones(N, device=DEV)
    p = ulorl.Params(gate_mode=ulorl.GATE_PER_RESPONSE, is_mode=ulorl.IS_POIS)   # paper's tau, sigma
    res = ulorl.token_loss_fwd(z, y, cu, adv, None, p)
    assert int(res.resp_gate[0]) == 1 and int(res.mpt_mask.sum()) == N
    assert res.loss.item() == 0.0 and torch.all(res.gcoef == 0)
    dz = ulorl.token_loss_bwd(z, y, res.lse, res.gcoef)
    assert torch.all(dz == 0)
    # negative advantage: same rows are never masked
    res2 = ulorl.token_loss_fwd(z, y, cu, -adv, None, p)
    assert int(res2.mpt_mask.sum()) == 0 and res2.loss.item() == 1.0
    assert int(res2.counters[2]) == 0


def test_exact_threshold_boundary_rows():
    """Spike rows just above / below p = tau (closed form a* = ln(99 (V-1)))."""
    import math
    V = 4096
    a_star = math.log(99 * (V - 1))
    z = torch.zeros(4, V, device=DEV)
    for t, da in enumerate([+3e-4, -3e-4, +3e-4, -3e-4]):
        z[t, 100 + t] = a_star + da
    y = torch.tensor([100, 101, 102, 103], dtype=torch.int32, device=DEV)
    cu = torch.tensor([0, 4], dtype=torch.int32, device=DEV)
    adv = torch.tensor([1.0, 1.0, -1.0, 1.0], device=DEV)
    p = ulorl.Params(gate_mode=ulorl.GATE_ALWAYS, is_mode=ulorl.IS_POIS)
    res = ulorl.token_loss_fwd(z, y, cu, adv, None, p)
    lse, logp, H = oracle.row_stats(z.cpu().numpy(), y.cpu().numpy())
    tt = oracle_terms(logp, H, [0, 4], adv.cpu().numpy(), None, p)
    assert np.all(np.abs(np.exp(logp) - f32(0.99)) > 1e-6)
    np.testing.assert_array_equal(res.mpt_mask.cpu().numpy(), tt.mask)
    assert list(tt.mask) == [1, 0, 0, 0]


def test_stats_only_pass_and_determinism():
    w = ui.shrink(ui.config(2), [333], V=20000, name="stats_only")
    d = ui.generate(w, DEV)
    a = ulorl.row_stats(d["logits"], d["token_ids"])
    b = ulorl.row_stats(d["logits"], d["token_ids"])
    assert a.loss is None and a.gcoef is None
    for x, yv in ((a.lse, b.lse), (a.logp, b.logp), (a.entropy, b.entropy)):
        assert torch.equal(x, yv)
    hl, y = _host(d)
    o = oracle.row_stats(hl, y)
    for name, g, r in zip(("lse", "logp", "entropy"), (a.lse, a.logp, a.entropy), o):
        assert_close(name, g.cpu().numpy(), r, rtol_for("bf16"))
    p = params_for(w, gate_mode=ulorl.GATE_ALWAYS)
    r1 = ulorl.token_loss_fwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    r2 = ulorl.token_loss_fwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    assert torch.equal(r1.loss, r2.loss) and torch.equal(r1.gcoef, r2.gcoef)
    z1 = ulorl.token_loss_bwd(d["logits"], d["token_ids"], r1.lse, r1.gcoef)
    z2 = ulorl.token_loss_bwd(d["logits"], d["token_ids"], r2.lse, r2.gcoef)
    assert torch.equal(z1.view(torch.int16), z2.view(torch.int16))


def test_explicit_segment_ids_pass_through():
    w = ui.shrink(ui.config(2), [50, 30], V=512, seg_len=16)
    d = ui.generate(w, DEV)
    ids = torch.arange(80, dtype=torch.int32, device=DEV).flip(0).contiguous()
    p = params_for(w, seg_len=0)
    res = ulorl.token_loss_fwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"],
                               d["old_logp"], p, segment_ids=ids)
    assert torch.equal(res.segment_out, ids)


def test_fused_path_defers_mpt_members_until_the_gate_is_known():
    """Under the entropy gates the one-call path finishes MPT members in a second launch; the
    result must not depend on which path produced it (checked against the oracle inside
    run_full_parity for every case above); here the deferred rows are the majority."""
    from dataclasses import replace
    w = replace(ui.shrink(ui.config(2), [300, 280, 310, 290], seg_len=100), spike_boost=22.0, spike_frac=0.7,
                name="cfg2_mostly_mpt")
    d = ui.generate(w, DEV)
    hl, y = _host(d)
    sigma = sigma_between_responses(hl, y, w.cu_seqlens)
    rows = np.arange(0, w.N, 11)
    for mode, sg in ((ulorl.GATE_PER_RESPONSE, sigma), (ulorl.GATE_GLOBAL, 100.0), (ulorl.GATE_GLOBAL, 0.0)):
        res, tt, _ = run_full_parity(w, params_for(w, gate_mode=mode, sigma=sg), dz_rows=rows, data=d)
    p = params_for(w, gate_mode=ulorl.GATE_PER_RESPONSE, sigma=sigma)
    res, tt, _ = run_full_parity(w, p, dz_rows=rows, data=d)
    assert 0 < tt.resp_gate.sum() < 4 and tt.n_masked > 100
    # device-detected errors behave the same through the one-call path
    ybad = d["token_ids"].clone()
    ybad[5] = w.V
    r1 = ulorl.token_loss_fwd(d["logits"], ybad, d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    z1 = ulorl.token_loss_bwd(d["logits"], ybad, r1.lse, r1.gcoef)
    r2, z2 = ulorl.token_loss_fwd_bwd(d["logits"], ybad, d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    assert int(r2.counters[3]) == ulorl.STATUS_BAD_TOKEN and torch.all(z2[5] == 0)
    # same gradient up to the rounding of the row sums (one bf16 ulp; the chosen column g - g p
    # cancels, hence the absolute term of a few 1e-6 |g|), zero rows identical
    assert torch.equal(z1 == 0, z2 == 0)
    gmax = float(r1.gcoef.abs().max())
    assert torch.all((z1.float() - z2.float()).abs() <= 2.0 ** -7 * z1.float().abs() + 8e-6 * gmax)
    cu_bad = d["cu_seqlens"].clone()
    cu_bad[1] = 700
    r3, z3 = ulorl.token_loss_fwd_bwd(d["logits"], d["token_ids"], cu_bad, d["advantages"], d["old_logp"], p)
    assert int(r3.counters[3]) & ulorl.STATUS_BAD_CU and torch.all(z3 == 0) and r3.loss.item() == 0.0


# ------------------------------------------------------------------ masked vocabulary entries

@pytest.mark.parametrize("dtype,V", [("bf16", 30011), ("f32", 9001)])
def test_rows_with_minus_infinity_logits_are_reported_not_trained(dtype, V):
    """Logits of -infinity are outside the domain (the oracle takes them as probability 0; the
    kernels' entropy sum turns not-a-number): such rows are reported through the status word and get
    a zero gradient on both paths; the other rows are untouched."""
    base = ui.config(1) if dtype == "f32" else ui.config(2)
    w = ui.shrink(base, [17, 5, 31], V=V, seg_len=8, name="masked_vocab_%s" % dtype)
    d = ui.generate(w, DEV)
    p = params_for(w, gate_mode=ulorl.GATE_ALWAYS, tau=0.5)
    vec = 4 if dtype == "f32" else 8
    stride = (V + vec - 1) // vec * vec                                   # rows padded to 16 bytes
    buf = torch.full((w.N, stride), float("nan"), dtype=w.torch_dtype(), device=DEV)
    buf[:, :V] = d["logits"]
    z = buf[:, :V]
    args = (d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    good = ulorl.token_loss_fwd(z, *args)
    assert int(good.counters[3]) == 0
    rows = [4, 20]
    for t in rows:
        cols = torch.arange(3 + t, V, 97, device=DEV)
        cols = cols[cols != d["token_ids"][t]]
        z[t, cols] = float("-inf")
    r = ulorl.token_loss_fwd(z, *args)
    dz = ulorl.token_loss_bwd(z, d["token_ids"], r.lse, r.gcoef)
    r1, dz1 = ulorl.token_loss_fwd_bwd(z, *args)
    other = torch.ones(w.N, dtype=torch.bool, device=DEV)
    other[rows] = False
    for res, grad in ((r, dz), (r1, dz1)):
        assert int(res.counters[3]) == ulorl.STATUS_NONFINITE
        assert torch.all(res.gcoef[rows] == 0) and torch.all(grad[rows] == 0)
        # the denominator is unchanged, so the other rows' coefficients are too
        assert torch.equal(res.gcoef[other], good.gcoef[other])
    assert torch.equal(_int_view(dz), _int_view(dz1))


def _int_view(t):
    return t.contiguous().view(torch.int32 if t.dtype == torch.float32 else torch.int16)


# ------------------------------------------------------------------ errors the device reports

def test_device_detected_errors_raise_status_bits_without_faulting():
    w = ui.shrink(ui.config(1), [20, 12], V=300, seg_len=8)
    d = ui.generate(w, DEV)
    p = params_for(w, gate_mode=ulorl.GATE_NEVER)
    good = ulorl.token_loss_fwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    assert int(good.counters[3]) == 0

    y = d["token_ids"].clone()
    y[3] = 300
    y[7] = -1
    r = ulorl.token_loss_fwd(d["logits"], y, d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    assert int(r.counters[3]) == ulorl.STATUS_BAD_TOKEN
    assert r.gcoef[3].item() == 0.0 and r.gcoef[7].item() == 0.0
    ok = torch.ones(32, dtype=torch.bool, device=DEV)
    ok[3] = ok[7] = False
    assert torch.equal(r.gcoef[ok], good.gcoef[ok])
    dz = ulorl.token_loss_bwd(d["logits"], y, r.lse, r.gcoef)
    assert torch.all(dz[3] == 0) and torch.all(dz[7] == 0)

    z = d["logits"].clone()
    z[5, 11] = float("inf")
    z[6, 12] = float("nan")
    r = ulorl.token_loss_fwd(z, d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    assert int(r.counters[3]) == ulorl.STATUS_NONFINITE
    assert r.gcoef[5].item() == 0.0 and r.gcoef[6].item() == 0.0
    assert torch.isfinite(r.loss).all()

    for bad in ([0, 25, 20, 32], [1, 20, 32], [0, 20, 31], [0, 20, 40]):
        cu = torch.tensor(bad, dtype=torch.int32, device=DEV)
        r = ulorl.token_loss_fwd(d["logits"], d["token_ids"], cu, d["advantages"], d["old_logp"], p)
        assert int(r.counters[3]) & ulorl.STATUS_BAD_CU
        assert r.loss.item() == 0.0 and torch.all(r.gcoef == 0)


@pytest.mark.parametrize("lengths", [[1], [1023, 1, 1025], [3] * 700, [2049]])
def test_workspace_and_outputs_are_never_overrun(lengths):
    """Guard bytes behind the workspace, the per-token outputs and the gradient stay untouched by
    the two-call and the one-call path (token counts around the 1024-token block of the O(N)
    kernels, many tiny responses)."""
    w = ui.shrink(ui.config(2), lengths, V=1000, seg_len=7, name="guard")
    d = ui.generate(w, DEV)
    p = params_for(w, gate_mode=ulorl.GATE_PER_RESPONSE, sigma=6.0)
    need = ulorl.token_loss_workspace_bytes(w.N, w.V, w.R)
    guard = 1 << 16
    buf = torch.full((need + guard,), 0xA5, dtype=torch.uint8, device=DEV)
    dz_buf = torch.full((w.N * w.V + guard,), -3.0, dtype=torch.bfloat16, device=DEV)
    dz = dz_buf[:w.N * w.V].view(w.N, w.V)
    out = ulorl.token_loss_fwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p,
                               workspace=buf[:need])
    ulorl.token_loss_bwd(d["logits"], d["token_ids"], out.lse, out.gcoef, 1.0, dlogits=dz)
    ulorl.token_loss_fwd_bwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p,
                             grad_out=1.0, dlogits=dz, out=out, workspace=buf[:need])
    torch.cuda.synchronize()
    assert bool((buf[need:] == 0xA5).all())
    assert bool((dz_buf[w.N * w.V:] == -3.0).all())


@pytest.mark.parametrize("gate", ["always", "per_response"])
@pytest.mark.parametrize("inplace", [False, True])
def test_an_expired_wait_costs_time_not_data(gate, inplace):
    """The workgroups that share a row wait for each other with a bounded wait.  With the bound set
    to a single poll from the host, many waits expire: the kernel still ends, the status word says
    so, and the repair pass finishes those rows -- every output and every gradient carries the bits
    of an undisturbed call, in place too (an expired workgroup has written nothing, so its piece of
    the logits was still intact)."""
    w = ui.shrink(ui.config(2), [400, 240], V=151936 // 2, name="sync_expiry")     # several pieces per row
    d = ui.generate(w, DEV)
    if gate == "always":
        p = params_for(w, gate_mode=ulorl.GATE_ALWAYS, tau=0.5)
    else:       # one response gated, one not: deferred rows and expired pieces meet
        hl, y = _host(d)
        p = params_for(w, gate_mode=ulorl.GATE_PER_RESPONSE, tau=0.5, sigma=sigma_between_responses(hl, y, w.cu_seqlens))
    args = (d["token_ids"], d["cu_seqlens"], d["advantages"], d["old_logp"], p)
    good, dz_good = ulorl.token_loss_fwd_bwd(d["logits"], *args)
    assert int(good.counters[3].item()) == 0
    if gate == "always":
        assert int(good.counters[0].item()) > 0
    seen = 0
    for attempt in range(4):        # a single poll nearly always expires somewhere among 3200 workgroups
        z = d["logits"].clone() if inplace else d["logits"]
        res, dz = ulorl.token_loss_fwd_bwd(z, *args, inplace=inplace, launch=ulorl.Launch(sync_spins=1))
        torch.cuda.synchronize()
        status = int(res.counters[3].item())
        assert status in (0, ulorl.STATUS_SYNC)         # 0: every partner happened to be there at the first poll
        seen += status == ulorl.STATUS_SYNC
        for name in ("loss", "logp", "entropy", "lse", "gcoef", "mpt_mask", "ratio", "segment_out", "resp_entropy",
                     "resp_gate"):
            assert torch.equal(getattr(res, name), getattr(good, name)), name
        assert torch.equal(res.counters[:3], good.counters[:3])
        assert torch.equal(dz.view(torch.int16), dz_good.view(torch.int16))
        if inplace:
            assert dz.data_ptr() == z.data_ptr()
        if seen:
            break
    assert seen, "no wait expired in four calls with a single poll: the repair pass was not exercised"


def test_rows_too_long_for_the_cooperative_kernel_fall_back():
    """A row of more than 64 pieces (1.97 M bf16 logits) is handled by one looping workgroup per
    row; a row of exactly 64 pieces still takes the cooperative kernel.  Both against the oracle."""
    for V in (64 * 3840 * 8, 64 * 3840 * 8 + 8):
        w = ui.shrink(ui.config(2), [2, 1], V=V, seg_len=1, name="long_rows_%d" % V)
        run_full_parity(w, params_for(w, gate_mode=ulorl.GATE_ALWAYS))
