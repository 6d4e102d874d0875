"""Shared machinery of the GPU-vs-oracle parity tests: run the HIP path through the C ABI,
run the fp64 oracle on the same seeded inputs, compare element by element.

Tolerances:
  * integer / byte outputs (MPT mask, segment ids, gates, counters): bit-exact, except that
    tokens whose oracle probability lies within 1e-6 of tau (mask) or whose ratio lies within
    1e-5 of a clip edge (clip counter) are excluded -- both are discontinuities.
  * per-row floats computed in fp32 from exact inputs (lse, logp, entropy, ratio, gcoef, loss):
    |gpu - ref| <= RTOL*|ref| + ATOL with RTOL = 1e-5 for fp32 logits and 2e-5 for bf16 logits
    (far inside the 2e-3 asked for bf16), ATOL = 2e-6 (the resolution of fp32 logits of
    magnitude 16-32, which bounds any difference of two of them).
  * dlogits: fp32 storage RTOL*|ref| + 4e-6*|g_t|; bf16 storage additionally half a bf16 ulp,
    2^-8*|ref| (round-to-nearest-even of the fp32 value).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2507_19766_amd as ulorl
import ulorl_inputs as ui

ATOL = 2e-6


def rtol_for(dtype: str) -> float:
    return 1e-5 if dtype == "f32" else 2e-5


def assert_close(name, got, ref, rtol, atol=ATOL):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    err = np.abs(got - ref)
    bound = rtol * np.abs(ref) + atol
    bad = ~(err <= bound)
    if bad.any():
        k = int(np.argmax(err - bound))
        raise AssertionError("%s: %d/%d outside tolerance; worst at %d: gpu=%r ref=%r err=%.3e bound=%.3e"
                             % (name, bad.sum(), bad.size, k, got.flat[k], ref.flat[k], err.flat[k], bound.flat[k]))


def params_for(w: ui.Workload, **kw) -> ulorl.Params:
    base = dict(eps_low=w.eps_low, eps_high=w.eps_high, tau=w.tau, sigma=w.sigma, seg_len=w.seg_len)
    base.update(kw)
    return ulorl.Params(**base)


def f32(x: float) -> float:
    """The double value of x after the float32 rounding the C struct applies."""
    return float(np.float32(x))


def oracle_terms(logp, ent, cu, adv, old, p: ulorl.Params, denominator=None, segment_ids=None):
    return oracle.token_terms(
        logp, ent, cu, adv, old, segment_ids=segment_ids, seg_len=p.seg_len,
        eps_low=f32(p.eps_low), eps_high=f32(p.eps_high), tau=f32(p.tau), sigma=f32(p.sigma),
        is_mode=p.is_mode, gate_mode=p.gate_mode,
        denominator=p.denominator if denominator is None else denominator)


def check_token_outputs(res: ulorl.FwdResult, tt, o_logp, p: ulorl.Params, rtol, rows=None,
                        check_counters=True):
    """Per-token outputs of the forward call against the oracle's token terms."""
    sel = slice(None) if rows is None else rows
    g_mask = res.mpt_mask.cpu().numpy()[sel]
    g_ratio = res.ratio.cpu().numpy()[sel]
    g_g = res.gcoef.cpu().numpy()[sel]
    prob = np.exp(o_logp)
    near_tau = np.abs(prob - f32(p.tau)) < 1e-6
    near_edge = (np.abs(tt.ratio - (1 - f32(p.eps_low))) < 1e-5) | (np.abs(tt.ratio - (1 + f32(p.eps_high))) < 1e-5)
    ok_m = ~near_tau
    np.testing.assert_array_equal(g_mask[ok_m], tt.mask[ok_m], err_msg="MPT mask")
    assert_close("ratio", g_ratio, tt.ratio, rtol, atol=0.0)
    ok_g = ok_m & ~near_edge
    assert_close("gcoef", g_g[ok_g], tt.gcoef[ok_g], rtol, atol=0.0)
    # exact zeros where the oracle has exact zeros
    assert np.all(g_g[ok_g][tt.gcoef[ok_g] == 0.0] == 0.0)
    if check_counters and rows is None:
        cnt = res.counters.cpu().numpy()
        assert abs(int(cnt[0]) - tt.n_masked) <= int(near_tau.sum())
        assert abs(int(cnt[1]) - tt.n_clip_inactive) <= int(near_edge.sum())
        assert int(cnt[2]) == tt.n_pos
        assert int(cnt[3]) == 0
    return int(near_tau.sum()), int(near_edge.sum())


def dlogits_bound(ref, g_rows, dtype: str, rtol):
    b = rtol * np.abs(ref) + 4e-6 * np.abs(g_rows)[:, None]
    if dtype == "bf16":
        b = b + 2.0 ** -8 * np.abs(ref)
    return b


def check_dlogits(name, got_rows: torch.Tensor, ref, g_rows, dtype, rtol):
    got = got_rows.detach().float().cpu().numpy().astype(np.float64)
    err = np.abs(got - ref)
    bound = dlogits_bound(ref, g_rows, dtype, rtol)
    bad = ~(err <= bound)
    if bad.any():
        k = np.unravel_index(int(np.argmax(err - bound)), err.shape)
        raise AssertionError("%s dlogits: %d outside tolerance; worst at %s gpu=%r ref=%r g=%r"
                             % (name, bad.sum(), k, got[k], ref[k], g_rows[k[0]]))
    zero_rows = g_rows == 0.0
    assert np.all(got[zero_rows] == 0.0), "rows with zero coefficient must be exactly zero"


def check_forward_against_oracle(res: ulorl.FwdResult, o_lse, o_logp, o_H, tt, p: ulorl.Params, rtol, loss_slack_rows=0):
    """Every per-row, per-token and per-response output of a forward (or one-call) result against
    the oracle's.  Returns (tokens near tau, tokens near a clip edge)."""
    assert_close("lse", res.lse.cpu().numpy(), o_lse, rtol)
    assert_close("logp", res.logp.cpu().numpy(), o_logp, rtol)
    assert_close("entropy", res.entropy.cpu().numpy(), o_H, rtol)
    np.testing.assert_array_equal(res.segment_out.cpu().numpy(), tt.seg)
    assert_close("resp_entropy", res.resp_entropy.cpu().numpy(), tt.resp_entropy, rtol)
    np.testing.assert_array_equal(res.resp_gate.cpu().numpy(), tt.resp_gate)
    n_tau, n_edge = check_token_outputs(res, tt, o_logp, p, rtol)
    if n_tau == 0 and n_edge == 0:
        assert_close("loss", res.loss.cpu().numpy()[0], tt.loss, rtol, atol=1e-7)
    elif loss_slack_rows:   # a token on a discontinuity may legitimately differ: bound its effect on the mean
        assert abs(res.loss.item() - tt.loss) <= rtol * abs(tt.loss) + 2.0 * (n_tau + n_edge) / loss_slack_rows
    return n_tau, n_edge


def near_discontinuity(o_logp, tt, p: ulorl.Params):
    return (np.abs(np.exp(o_logp) - f32(p.tau)) < 1e-6) | \
           (np.abs(tt.ratio - (1 - f32(p.eps_low))) < 1e-5) | (np.abs(tt.ratio - (1 + f32(p.eps_high))) < 1e-5)


def run_full_parity(w: ui.Workload, p: ulorl.Params, dz_rows=None, inplace=False, data=None,
                    grad_out=1.0, same_bits=True):
    """Whole path on the GPU vs whole oracle on the host, every row: the two-call path, then (when
    the logits survive, i.e. not in place) the one-call path in both of its kernels.
    ``same_bits``: the two-call forward runs by pieces (the library's default), so the two paths
    must agree bit for bit.  Returns (res, tt, info)."""
    dev = torch.device("cuda:0")
    d = data if data is not None else ui.generate(w, dev)
    logits = d["logits"]
    old = None if p.is_mode == ulorl.IS_POIS else d["old_logp"]
    res = ulorl.token_loss_fwd(logits, d["token_ids"], d["cu_seqlens"], d["advantages"], old, p)
    host_logits = ui.to_numpy_logits(logits)
    y = d["token_ids"].cpu().numpy()
    rtol = rtol_for(w.dtype)

    o_lse, o_logp, o_H = oracle.row_stats(host_logits, y)
    adv = d["advantages"].cpu().numpy()
    oldh = None if old is None else old.cpu().numpy()
    tt = oracle_terms(o_logp, o_H, w.cu_seqlens, adv, oldh, p)
    n_tau, n_edge = check_forward_against_oracle(res, o_lse, o_logp, o_H, tt, p, rtol)

    rows = np.arange(w.N) if dz_rows is None else np.asarray(dz_rows)
    # the oracle's gradient uses the oracle's own lse and coefficient
    ref = oracle.dlogits(host_logits, y, o_lse, tt.gcoef, grad_out=grad_out, rows=rows)
    keep = ~near_discontinuity(o_logp, tt, p)[rows]
    sel = torch.as_tensor(rows[keep], device=dev)

    def compare_dz(name, dz_tensor):
        check_dlogits(name, dz_tensor[sel], ref[keep], grad_out * tt.gcoef[rows][keep], w.dtype, rtol)

    pristine = None if inplace else logits
    dz1 = None
    if not inplace:     # the one-call path first, while the logits are intact
        dz1 = check_one_call_path(d, p, res, o_lse, o_logp, o_H, tt, rtol, compare_dz, grad_out=grad_out,
                                  same_bits=same_bits)
    dz = ulorl.token_loss_bwd(logits, d["token_ids"], res.lse, res.gcoef, grad_out=grad_out,
                              inplace=inplace)
    compare_dz(w.name, dz)
    if dz1 is not None and same_bits:
        assert torch.equal(_bits(dz1), _bits(dz)), "one-call dlogits differ from the two-call dlogits"
    if pristine is not None:
        check_row_kernels_bitwise(d, p, grad_out=grad_out)
    return res, tt, dict(n_near_tau=n_tau, n_near_edge=n_edge, dz=dz, data=d, o_H=o_H)


def _bits(t: torch.Tensor) -> torch.Tensor:
    if t.dtype == torch.float32:
        return t.view(torch.int32)
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16)
    return t


def assert_same_results(a: ulorl.FwdResult, b: ulorl.FwdResult, what=""):
    for name in ("loss", "logp", "entropy", "lse", "gcoef", "mpt_mask", "ratio", "segment_out", "resp_entropy",
                 "resp_gate", "counters"):
        x, yv = getattr(a, name), getattr(b, name)
        assert torch.equal(_bits(x), _bits(yv)), "%s: %s differs between the fused and the two-call path" % (what, name)


def check_one_call_path(d, p: ulorl.Params, res2: ulorl.FwdResult, o_lse, o_logp, o_H, tt, rtol, compare_dz,
                        grad_out=1.0, also_inplace=True, same_bits=True):
    """The one-call forward+backward (row-cooperative kernel) against the oracle, out of place and
    (on a copy of the logits) in place; and against the two-call result: the same bits when the
    two-call forward ran by pieces, else the same integer decisions wherever the oracle is not on
    a discontinuity.  Returns the out-of-place dlogits."""
    old = None if p.is_mode == ulorl.IS_POIS else d["old_logp"]
    r1, dz1 = ulorl.token_loss_fwd_bwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], old, p,
                                       grad_out=grad_out)
    check_forward_against_oracle(r1, o_lse, o_logp, o_H, tt, p, rtol)
    compare_dz("one-call", dz1)
    assert int(r1.counters[3].item()) & ulorl.STATUS_SYNC == 0
    far = torch.as_tensor(~near_discontinuity(o_logp, tt, p), device=r1.mpt_mask.device)
    assert torch.equal(r1.mpt_mask[far], res2.mpt_mask[far])
    assert torch.equal((r1.gcoef == 0)[far], (res2.gcoef == 0)[far])
    assert torch.equal(r1.resp_gate, res2.resp_gate) and torch.equal(r1.segment_out, res2.segment_out)
    if same_bits:
        assert_same_results(res2, r1, "one call vs two calls")
    if also_inplace and d["logits"].is_contiguous():
        z = d["logits"].clone()
        r3, dz3 = ulorl.token_loss_fwd_bwd(z, d["token_ids"], d["cu_seqlens"], d["advantages"], old, p,
                                           grad_out=grad_out, inplace=True)
        assert dz3.data_ptr() == z.data_ptr()
        assert_same_results(r1, r3, "in place")
        assert torch.equal(_bits(dz3), _bits(dz1)), "one-call in-place dlogits differ from out-of-place"
    return dz1


def check_row_kernels_bitwise(d, p: ulorl.Params, grad_out=1.0):
    """The kernels with one looping workgroup per row (the fallbacks of both paths) reproduce each
    other bit for bit as well."""
    old = None if p.is_mode == ulorl.IS_POIS else d["old_logp"]
    ulorl.tune(ulorl.TUNE_FUSED_CLUSTER, 0)
    ulorl.tune(ulorl.TUNE_FWD_PIECES, 0)
    try:
        r2, dz2 = ulorl.token_loss_fwd_bwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], old, p,
                                           grad_out=grad_out)
        res = ulorl.token_loss_fwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], old, p)
        dz = ulorl.token_loss_bwd(d["logits"], d["token_ids"], res.lse, res.gcoef, grad_out=grad_out)
    finally:
        ulorl.tune(ulorl.TUNE_FUSED_CLUSTER, 1)
        ulorl.tune(ulorl.TUNE_FWD_PIECES, 1)
    assert_same_results(res, r2, "row kernels")
    assert torch.equal(_bits(dz2), _bits(dz)), "row-kernel fused dlogits differ from the two-call dlogits"


def sigma_between_responses(host_logits, y, cu, k=None):
    """A target entropy midway between two responses' mean entropies (oracle side only), so that
    some responses are gated and others are not; asserts a margin of 1e-3 nats."""
    _, _, H = oracle.row_stats(host_logits, y)
    hbar = np.array([H[cu[i]:cu[i + 1]].mean() for i in range(len(cu) - 1) if cu[i + 1] > cu[i]])
    s = np.sort(hbar)
    gaps = np.diff(s)
    j = int(np.argmax(gaps)) if k is None else k
    assert gaps[j] > 2e-3, "responses' mean entropies too close for a gate test"
    return 0.5 * (s[j] + s[j + 1])


def oracle_row_stats_streamed(logits: torch.Tensor, y_host: np.ndarray, block_rows=4096, keep_rows=None,
                              progress=None):
    """Oracle row statistics of a device tensor of any size: rows are copied to the host block by
    block (the host never holds the whole tensor).  Optionally keeps host copies of a few rows."""
    N = logits.shape[0]
    lse = np.empty(N)
    logp = np.empty(N)
    ent = np.empty(N)
    kept = {}
    keep = set(int(r) for r in (keep_rows if keep_rows is not None else []))
    for r0 in range(0, N, block_rows):
        r1 = min(N, r0 + block_rows)
        host = ui.to_numpy_logits(logits[r0:r1])
        lse[r0:r1], logp[r0:r1], ent[r0:r1] = oracle.row_stats(host, y_host[r0:r1])
        for r in keep:
            if r0 <= r < r1:
                kept[r] = host[r - r0].copy()
        if progress:
            progress(r1, N)
    return lse, logp, ent, kept


def run_streamed_parity(w: ui.Workload, p: ulorl.Params, data, n_dz_rows=64, inplace=True, seed=0,
                        say=print, one_call=False):
    """Full-size parity: every row's statistics and every token's terms against the oracle (logits
    streamed to the host in blocks, before anything overwrites them), the gradient on sampled
    rows.  one_call selects ulorl_token_loss_fwd_bwd instead of the forward / backward pair."""
    dev = data["logits"].device
    logits = data["logits"]
    rtol = rtol_for(w.dtype)
    y = data["token_ids"].cpu().numpy()
    adv = data["advantages"].cpu().numpy()
    old = None if p.is_mode == ulorl.IS_POIS else data["old_logp"]

    rs = np.random.RandomState(seed)
    rows = np.unique(np.concatenate([[0, w.N - 1], rs.choice(w.N, n_dz_rows, replace=False)]))
    say("streaming %d rows to the oracle" % w.N)
    o_lse, o_logp, o_H, kept = oracle_row_stats_streamed(
        logits, y, keep_rows=rows,
        progress=lambda a, b: say("  oracle rows %d/%d" % (a, b)) if (a // 4096) % 8 == 0 or a == b else None)
    tt = oracle_terms(o_logp, o_H, w.cu_seqlens, adv, None if old is None else old.cpu().numpy(), p)

    if one_call:
        res, dz = ulorl.token_loss_fwd_bwd(logits, data["token_ids"], data["cu_seqlens"], data["advantages"], old, p,
                                           inplace=inplace)
    else:
        res = ulorl.token_loss_fwd(logits, data["token_ids"], data["cu_seqlens"], data["advantages"], old, p)
        dz = ulorl.token_loss_bwd(logits, data["token_ids"], res.lse, res.gcoef, inplace=inplace)
    torch.cuda.synchronize()
    say("%s done" % ("one call" if one_call else "forward + backward"))
    n_tau, n_edge = check_forward_against_oracle(res, o_lse, o_logp, o_H, tt, p, rtol, loss_slack_rows=w.N)
    say("token terms ok (masked %d, clipped %d, near tau %d, near clip edge %d)"
        % (tt.n_masked, tt.n_clip_inactive, n_tau, n_edge))

    near = near_discontinuity(o_logp, tt, p)
    rows = np.array([r for r in rows if not near[r]])
    sub = np.stack([kept[int(r)] for r in rows])
    ref = oracle.dlogits(sub, y[rows], o_lse[rows], tt.gcoef[rows])
    check_dlogits(w.name, dz[torch.as_tensor(rows, device=dev)], ref, tt.gcoef[rows], w.dtype, rtol)
    # properties that hold at any size: masked / clipped rows are exactly zero
    zero_rows = np.nonzero(tt.gcoef == 0.0)[0]
    zero_rows = zero_rows[~near[zero_rows]][:256]
    if len(zero_rows):
        assert torch.all(dz[torch.as_tensor(zero_rows, device=dev)] == 0)
    say("dlogits ok on %d sampled rows, %d zero rows" % (len(rows), len(zero_rows)))
    return res, tt


# ------------------------------------------------------------------------------------ lm_head variant

LMHEAD_ATOL = 4e-6   # fp32 MFMA accumulation of Hd ~ 2048 products adds ~1e-6 to every logit


def raw_bf16(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def run_lmhead_parity(w: ui.Workload, p: ulorl.Params, chunk: int, data=None, grad_out=1.0, say=None):
    """lm_head variant through the C ABI against the oracle (fp64 logits from a stock matrix
    product, then the same oracle functions as the logits path, then the chain rule to hidden, W)."""
    dev = torch.device("cuda:0")
    d = data if data is not None else ui.generate(w, dev)
    hidden, weight = d["hidden"], d["weight"]
    old = None if p.is_mode == ulorl.IS_POIS else d["old_logp"]
    res = ulorl.lmhead_token_loss_fwd(hidden, weight, d["token_ids"], d["cu_seqlens"], d["advantages"], old, p,
                                      vocab_chunk=chunk)
    dH, dW = ulorl.lmhead_token_loss_bwd(hidden, weight, d["token_ids"], res.lse, res.gcoef, grad_out=grad_out,
                                         vocab_chunk=chunk)
    torch.cuda.synchronize()
    if say:
        say("gpu done; oracle logits %d x %d x %d" % (w.N, w.hidden, w.V))
    hr, wr = raw_bf16(hidden), raw_bf16(weight)
    z = oracle.lmhead_logits(hr, wr)
    y = d["token_ids"].cpu().numpy()
    rtol = rtol_for("bf16")
    o_lse, o_logp, o_H = oracle.row_stats(z, y)
    assert_close("lse", res.lse.cpu().numpy(), o_lse, rtol, atol=LMHEAD_ATOL)
    assert_close("logp", res.logp.cpu().numpy(), o_logp, rtol, atol=LMHEAD_ATOL)
    assert_close("entropy", res.entropy.cpu().numpy(), o_H, rtol, atol=LMHEAD_ATOL)
    adv = d["advantages"].cpu().numpy()
    tt = oracle_terms(o_logp, o_H, w.cu_seqlens, adv, None if old is None else old.cpu().numpy(), p)
    np.testing.assert_array_equal(res.segment_out.cpu().numpy(), tt.seg)
    assert_close("resp_entropy", res.resp_entropy.cpu().numpy(), tt.resp_entropy, rtol, atol=LMHEAD_ATOL)
    np.testing.assert_array_equal(res.resp_gate.cpu().numpy(), tt.resp_gate)
    # same discontinuity exclusions as the logits path; the ratio inherits the logits' absolute error
    prob = np.exp(o_logp)
    near = (np.abs(prob - f32(p.tau)) < 2e-5) | (np.abs(tt.ratio - (1 - f32(p.eps_low))) < 2e-5) | \
           (np.abs(tt.ratio - (1 + f32(p.eps_high))) < 2e-5)
    np.testing.assert_array_equal(res.mpt_mask.cpu().numpy()[~near], tt.mask[~near])
    assert_close("ratio", res.ratio.cpu().numpy(), tt.ratio, 3e-5, atol=0.0)
    assert_close("gcoef", res.gcoef.cpu().numpy()[~near], tt.gcoef[~near], 3e-5, atol=0.0)
    if not near.any():
        assert_close("loss", res.loss.item(), tt.loss, 3e-5, atol=1e-7)
    assert int(res.counters[3]) == 0 and int(res.counters[2]) == tt.n_pos
    if say:
        say("forward ok; oracle gradients")

    g = tt.gcoef.copy()
    g[near] = res.gcoef.cpu().numpy()[near]      # a token on a discontinuity: take the GPU's side of it
    dz = oracle.dlogits(z, y, o_lse, g, grad_out=grad_out)
    rdH, rdW = oracle.lmhead_grads(hr, wr, dz)
    absdz = np.abs(dz)
    wf, hf = oracle.bf16_to_f64(wr), oracle.bf16_to_f64(hr)
    bH = absdz @ np.abs(wf).T
    bW = np.abs(hf).T @ absdz
    # root-sum-square of the terms: what independent rounding errors of the terms add up to
    qH = np.sqrt((dz * dz) @ (wf * wf).T)
    qW = np.sqrt((hf * hf).T @ (dz * dz))
    # dz is rounded to bf16 as a GEMM operand (relative 2^-8 per term, worst case all aligned),
    # the result is rounded to bf16 once (2^-8 relative), fp32 accumulation is negligible beside both
    for name, got, ref, bound, rss in (("d_hidden", dH, rdH, bH, qH), ("d_W", dW, rdW, bW, qW)):
        got = got.float().cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        tol = 2.0 ** -8 * bound + 2.0 ** -8 * np.abs(ref) + 1e-12
        bad = err > tol
        if bad.any():
            k = np.unravel_index(int(np.argmax(err - tol)), err.shape)
            raise AssertionError("%s: %d outside tolerance; worst at %s gpu=%r ref=%r tol=%r"
                                 % (name, bad.sum(), k, got[k], ref[k], tol[k]))
        # The worst-case bound is loose by about the square root of the number of terms.  The
        # typical error must stay below what independent roundings give: a round-to-nearest bf16
        # error is at most 2^-8 relative and 2^-9 in the root mean square, so the terms contribute
        # at most 2^-9 * rss and the final rounding 2^-9 * |ref| (root mean square each; the mean
        # absolute error is below either).
        typical = 2.0 ** -9 * (rss + np.abs(ref))
        assert err.mean() <= typical.mean() + 1e-12, (name, err.mean(), typical.mean())
    return res, tt
