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
                    grad_out=1.0, same_bits=True, launch=None):
    """Whole path on the GPU vs whole oracle on the host, every row: the two-call path, then (when
    the logits survive, i.e. not in place) the one-call path in both of its kernels.
    ``same_bits``: the two-call forward runs by pieces (the library's default), so the two paths
    must agree bit for bit.  Returns (res, tt, info)."""
    dev = torch.device("cuda:0")
    d = data if data is not None else ui.generate(w, dev)
    logits = d["logits"]
    old = None if p.is_mode == ulorl.IS_POIS else d["old_logp"]
    res = ulorl.token_loss_fwd(logits, d["token_ids"], d["cu_seqlens"], d["advantages"], old, p, launch=launch)
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
    """The kernels with one looping workgroup per row (ULORL_LAUNCH_PER_ROW: the fallbacks of both
    paths) reproduce each other bit for bit as well."""
    old = None if p.is_mode == ulorl.IS_POIS else d["old_logp"]
    per_row = ulorl.Launch(per_row=True)
    r2, dz2 = ulorl.token_loss_fwd_bwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], old, p,
                                       grad_out=grad_out, launch=per_row)
    res = ulorl.token_loss_fwd(d["logits"], d["token_ids"], d["cu_seqlens"], d["advantages"], old, p, launch=per_row)
    dz = ulorl.token_loss_bwd(d["logits"], d["token_ids"], res.lse, res.gcoef, grad_out=grad_out)
    assert_same_results(res, r2, "row kernels")
    assert torch.equal(_bits(dz2), _bits(dz)), "row-kernel fused dlogits differ from the two-call dlogits"
    return res, dz


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


def assert_row_sums_vanish(dz: torch.Tensor, V: int, block_rows=4096):
    """sum_j dz[t, j] = g_t (1 - sum_j p_j) = 0: on the stored (rounded) gradient the sum must stay
    within V * 2^-9 * max_j |dz[t, j]| (bf16 storage: V roundings, each of at most half an ulp of the
    row's largest entry)."""
    assert dz.dtype == torch.bfloat16
    scale = 2.0 ** -9
    for r0 in range(0, dz.shape[0], block_rows):
        blk = dz[r0:r0 + block_rows]
        s = blk.sum(dim=1, dtype=torch.float64).abs()
        bound = V * scale * blk.abs().amax(dim=1).double()
        assert bool((s <= bound).all()), "row sums of dlogits: rows %d.." % r0


def assert_same_bits_blockwise(a: torch.Tensor, b: torch.Tensor, what: str, block_rows=8192):
    assert a.shape == b.shape and a.dtype == b.dtype
    for r0 in range(0, a.shape[0], block_rows):
        if not torch.equal(_bits(a[r0:r0 + block_rows]), _bits(b[r0:r0 + block_rows])):
            x, y = _bits(a[r0:r0 + block_rows]), _bits(b[r0:r0 + block_rows])
            bad = (x != y).any(dim=1).nonzero()[:4, 0] + r0
            raise AssertionError("%s: rows %s differ" % (what, bad.tolist()))


# ------------------------------------------------------------------------------------ lm_head variant

LMHEAD_ATOL = 4e-6   # fp32 MFMA accumulation of Hd ~ 2048 products adds ~1e-6 to every logit


LMHEAD_EDGE_BAND = 2e-5   # clip-edge band of the lm_head variant (the mask keeps 1e-6)
LMHEAD_CHOSEN_RTOL = 1e-5  # fp32 error of g p at the chosen column, relative to g


def lmhead_near(o_logp, tt, p: ulorl.Params):
    """(tokens within 1e-6 of tau, tokens within LMHEAD_EDGE_BAND of a clip edge), oracle side."""
    near_tau = np.abs(np.exp(o_logp) - f32(p.tau)) < 1e-6
    near_edge = (np.abs(tt.ratio - (1 - f32(p.eps_low))) < LMHEAD_EDGE_BAND) | \
                (np.abs(tt.ratio - (1 + f32(p.eps_high))) < LMHEAD_EDGE_BAND)
    return near_tau, near_edge


def raw_bf16(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def run_lmhead_parity(w: ui.Workload, p: ulorl.Params, chunk: int, data=None, grad_out=1.0, say=None, launch=None):
    """lm_head variant through the C ABI against the oracle (fp64 logits from a stock matrix
    product, then the same oracle functions as the logits path, then the chain rule to hidden, W)."""
    dev = torch.device("cuda:0")
    d = data if data is not None else ui.generate(w, dev)
    hidden, weight = d["hidden"], d["weight"]
    old = None if p.is_mode == ulorl.IS_POIS else d["old_logp"]
    res = ulorl.lmhead_token_loss_fwd(hidden, weight, d["token_ids"], d["cu_seqlens"], d["advantages"], old, p,
                                      vocab_chunk=chunk, launch=launch)
    dH, dW = ulorl.lmhead_token_loss_bwd(hidden, weight, d["token_ids"], res.lse, res.gcoef, grad_out=grad_out,
                                         vocab_chunk=chunk, launch=launch)
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
    # The MPT mask keeps the 1e-6 band of the logits path: near p = tau = 0.99 an error d in a logit
    # moves p by p (1 - p) d ~ 0.01 d, so the 4e-6 of the fp32 accumulation stay far inside it.  The
    # ratio e^(logp - old) inherits the logits' absolute error as a relative one (4e-6 x 1.2), hence
    # the wider band at the clip edges only.
    near_tau, near_edge = lmhead_near(o_logp, tt, p)
    near = near_tau | near_edge
    np.testing.assert_array_equal(res.mpt_mask.cpu().numpy()[~near_tau], tt.mask[~near_tau])
    assert_close("ratio", res.ratio.cpu().numpy(), tt.ratio, 3e-5, atol=0.0)
    g_gpu = res.gcoef.cpu().numpy()
    assert_close("gcoef", g_gpu[~near], tt.gcoef[~near], 3e-5, atol=0.0)
    assert np.all(g_gpu[~near][tt.gcoef[~near] == 0.0] == 0.0)         # masked / clipped: exactly zero
    if not near.any():
        assert_close("loss", res.loss.item(), tt.loss, 3e-5, atol=1e-7)
    cnt = res.counters.cpu().numpy()
    assert int(cnt[3]) == 0 and int(cnt[2]) == tt.n_pos
    assert abs(int(cnt[0]) - tt.n_masked) <= int(near_tau.sum())
    assert abs(int(cnt[1]) - tt.n_clip_inactive) <= int(near_edge.sum())
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
    # The chosen column is computed as g - g p: where p is close to 1 the result is much smaller than
    # the fp32 error of g p (logit 4e-6, lse 4e-6, exponent argument 2e-6: LMHEAD_CHOSEN_RTOL of g),
    # the same absolute term the logits path allows on dlogits.
    ag = np.abs(grad_out * g)
    sH = LMHEAD_CHOSEN_RTOL * ag[:, None] * np.abs(wf)[:, y].T                      # [N, Hd]
    sWt = np.zeros((wf.shape[1], hf.shape[1]))
    np.add.at(sWt, y, LMHEAD_CHOSEN_RTOL * ag[:, None] * np.abs(hf))                # [V, Hd]
    for name, got, ref, bound, rss, slack in (("d_hidden", dH, rdH, bH, qH, sH), ("d_W", dW, rdW, bW, qW, sWt.T)):
        got = got.float().cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        tol = 2.0 ** -8 * bound + 2.0 ** -8 * np.abs(ref) + slack + 1e-12
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
        typical = 2.0 ** -9 * (rss + np.abs(ref)) + slack
        assert err.mean() <= typical.mean() + 1e-12, (name, err.mean(), typical.mean())
    # a token with a zero coefficient (masked, clipped) contributes nothing: its dHidden row is exactly zero
    zero = torch.as_tensor((tt.gcoef == 0.0) & ~near, device=dH.device)
    assert bool((dH[zero] == 0).all()), "rows with a zero coefficient must have an exactly zero d_hidden"
    res.d_hidden, res.d_weight = dH, dW
    return res, tt


def run_lmhead_streamed_parity(w: ui.Workload, p: ulorl.Params, data, chunk=8192, block_rows=2048, n_cols=512,
                               seed=0, say=print):
    """lm_head variant at any size against the oracle, EVERY row and EVERY element of d_hidden and
    d_W: the oracle's fp64 logits are formed block of rows by block of rows (stock matrix product),
    each block goes through the oracle's row statistics, token terms and gradient, and the chain rule
    to hidden and W is accumulated in fp64.  Needs a gate that does not couple rows (ALWAYS / NEVER):
    then a token's terms depend on its own row and on the denominator only.
    Bounds: as in run_lmhead_parity, except that the worst-case sum |dz| . |W| (resp. |hidden| . |dz|)
    is replaced over the whole matrices by its Cauchy-Schwarz bound from row / column norms (no extra
    matrix product); the exact sums and the typical-error check are applied on n_cols sampled
    vocabulary columns of d_W."""
    assert p.gate_mode in (ulorl.GATE_ALWAYS, ulorl.GATE_NEVER)
    hidden, weight = data["hidden"], data["weight"]
    old_t = None if p.is_mode == ulorl.IS_POIS else data["old_logp"]
    res = ulorl.lmhead_token_loss_fwd(hidden, weight, data["token_ids"], data["cu_seqlens"], data["advantages"],
                                      old_t, p, vocab_chunk=chunk)
    dH, dW = ulorl.lmhead_token_loss_bwd(hidden, weight, data["token_ids"], res.lse, res.gcoef, vocab_chunk=chunk)
    torch.cuda.synchronize()
    say("gpu forward + backward done; oracle over %d rows in blocks of %d" % (w.N, block_rows))
    N, Hd, V = w.N, w.hidden, w.V
    D = p.denominator if p.denominator > 0 else float(N)
    rtol = rtol_for("bf16")
    wr = raw_bf16(weight)
    wd = oracle.bf16_to_f64(wr)
    w_norm = np.sqrt((wd * wd).sum(1))                        # |W[k, :]|
    y = data["token_ids"].cpu().numpy()
    adv = data["advantages"].cpu().numpy()
    old = None if old_t is None else old_t.cpu().numpy()
    g_lse, g_logp, g_H = res.lse.cpu().numpy(), res.logp.cpu().numpy(), res.entropy.cpu().numpy()
    g_mask, g_ratio, g_g = res.mpt_mask.cpu().numpy(), res.ratio.cpu().numpy(), res.gcoef.cpu().numpy()
    cols = np.sort(np.random.RandomState(seed).choice(V, n_cols, replace=False))
    ref_dW = np.zeros((Hd, V))
    bW = np.zeros((Hd, n_cols))
    qW = np.zeros((Hd, n_cols))
    dz_sq = np.zeros(V)
    h_sq = np.zeros(Hd)
    slack_Wt = np.zeros((V, Hd))          # chosen-column term of the d_W tolerance, transposed
    resp = np.repeat(np.arange(w.R), w.lengths)
    h_sum = np.zeros(w.R)
    loss = 0.0
    n_masked = n_clip = n_pos = n_tau = n_edge = 0
    for r0 in range(0, N, block_rows):
        r1 = min(N, r0 + block_rows)
        hb = oracle.bf16_to_f64(raw_bf16(hidden[r0:r1]))
        z = hb @ wd
        o_lse, o_logp, o_H = oracle.row_stats(z, y[r0:r1])
        assert_close("lse", g_lse[r0:r1], o_lse, rtol, atol=LMHEAD_ATOL)
        assert_close("logp", g_logp[r0:r1], o_logp, rtol, atol=LMHEAD_ATOL)
        assert_close("entropy", g_H[r0:r1], o_H, rtol, atol=LMHEAD_ATOL)
        tt = oracle_terms(o_logp, o_H, [0, r1 - r0], adv[r0:r1], None if old is None else old[r0:r1], p, denominator=D)
        near_tau, near_edge = lmhead_near(o_logp, tt, p)
        near = near_tau | near_edge
        np.testing.assert_array_equal(g_mask[r0:r1][~near_tau], tt.mask[~near_tau])
        assert_close("ratio", g_ratio[r0:r1], tt.ratio, 3e-5, atol=0.0)
        assert_close("gcoef", g_g[r0:r1][~near], tt.gcoef[~near], 3e-5, atol=0.0)
        assert np.all(g_g[r0:r1][~near][tt.gcoef[~near] == 0.0] == 0.0)
        np.add.at(h_sum, resp[r0:r1], o_H)
        loss += tt.loss
        n_masked += tt.n_masked; n_clip += tt.n_clip_inactive; n_pos += tt.n_pos
        n_tau += int(near_tau.sum()); n_edge += int(near_edge.sum())
        g = tt.gcoef.copy()
        g[near] = g_g[r0:r1][near]           # a token on a discontinuity: either side is admissible
        dz = oracle.dlogits(z, y[r0:r1], o_lse, g)
        del z
        blk_dH = dz @ wd.T
        got = dH[r0:r1].float().cpu().numpy().astype(np.float64)
        ag = np.abs(g)
        tol = 2.0 ** -8 * np.sqrt((dz * dz).sum(1))[:, None] * w_norm[None, :] + 2.0 ** -8 * np.abs(blk_dH) + \
            LMHEAD_CHOSEN_RTOL * ag[:, None] * np.abs(wd)[:, y[r0:r1]].T + 1e-12
        err = np.abs(got - blk_dH)
        if (err > tol).any():
            k = np.unravel_index(int(np.argmax(err - tol)), err.shape)
            raise AssertionError("d_hidden rows %d..: worst at %s gpu=%r ref=%r tol=%r" % (r0, k, got[k], blk_dH[k], tol[k]))
        assert err.mean() <= 3e-3 * np.abs(blk_dH).mean() + 1e-12
        assert np.all(got[(g == 0.0)] == 0.0)
        ref_dW += hb.T @ dz
        np.add.at(slack_Wt, y[r0:r1], LMHEAD_CHOSEN_RTOL * ag[:, None] * np.abs(hb))
        dz_sq += (dz * dz).sum(0)
        h_sq += (hb * hb).sum(0)
        dzc = dz[:, cols]
        bW += np.abs(hb).T @ np.abs(dzc)
        qW += (hb * hb).T @ (dzc * dzc)
        del dz
        say("  oracle rows %d/%d" % (r1, N))
    # per-response and whole-batch outputs
    assert_close("resp_entropy", res.resp_entropy.cpu().numpy(), h_sum / np.asarray(w.lengths), rtol, atol=LMHEAD_ATOL)
    expect_gate = np.full(w.R, 1 if p.gate_mode == ulorl.GATE_ALWAYS else 0, np.uint8)
    np.testing.assert_array_equal(res.resp_gate.cpu().numpy(), expect_gate)
    cnt = res.counters.cpu().numpy()
    assert int(cnt[3]) == 0 and int(cnt[2]) == n_pos
    assert abs(int(cnt[0]) - n_masked) <= n_tau and abs(int(cnt[1]) - n_clip) <= n_edge
    if n_tau == 0 and n_edge == 0:
        assert_close("loss", res.loss.item(), loss, 3e-5, atol=1e-7)
    else:
        assert abs(res.loss.item() - loss) <= 3e-5 * abs(loss) + 2.0 * (n_tau + n_edge) / D
    say("forward and d_hidden ok on every row (masked %d, clipped %d, near tau %d, near a clip edge %d)"
        % (n_masked, n_clip, n_tau, n_edge))
    # d_W, every element
    got = dW.float().cpu().numpy().astype(np.float64)
    err = np.abs(got - ref_dW)
    slack_W = slack_Wt.T
    tol = 2.0 ** -8 * np.sqrt(h_sq)[:, None] * np.sqrt(dz_sq)[None, :] + 2.0 ** -8 * np.abs(ref_dW) + slack_W + 1e-12
    if (err > tol).any():
        k = np.unravel_index(int(np.argmax(err - tol)), err.shape)
        raise AssertionError("d_W: %d outside tolerance; worst at %s gpu=%r ref=%r tol=%r"
                             % ((err > tol).sum(), k, got[k], ref_dW[k], tol[k]))
    ec, rc = err[:, cols], np.abs(ref_dW[:, cols])
    tight = 2.0 ** -8 * bW + 2.0 ** -8 * rc + slack_W[:, cols] + 1e-12
    assert np.all(ec <= tight), "d_W on sampled columns: exact worst-case bound"
    typical = 2.0 ** -9 * (np.sqrt(qW) + rc) + slack_W[:, cols]
    assert ec.mean() <= typical.mean() + 1e-12, (ec.mean(), typical.mean())
    say("d_W ok on every element (mean error %.3e, mean magnitude %.3e; %d columns with exact bounds)"
        % (err.mean(), np.abs(ref_dW).mean(), n_cols))
    res.d_hidden, res.d_weight = dH, dW
    return res, dict(loss=loss, n_masked=n_masked, n_clip=n_clip, n_pos=n_pos)
