"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: ulorl_oracle.c is compiled
with -fsanitize=address,undefined into a small driver (oracle/sanitize_driver.c) whose buffers have
exactly the sizes the oracle's contract states, the driver runs every oracle entry point on edge-case
inputs (a vocabulary that is not a multiple of anything, padded rows whose last row ends at V, an
empty response, a response of one token, -inf logits, explicit segment ids outside the counted range,
all three storage types), and its results must equal those of the regular library.  CPU only."""
import os
import subprocess

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.join(os.path.dirname(HERE), "oracle")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("sanitized") / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           os.path.join(ORACLE_DIR, "ulorl_oracle.c"), os.path.join(ORACLE_DIR, "sanitize_driver.c"), "-o", exe, "-lm"]
    subprocess.check_call(cmd)
    return exe


def _case(seed, storage, lengths, V, pad, use_seg, use_old, is_mode, gate_mode, G):
    rs = np.random.RandomState(seed)
    N, R = int(sum(lengths)), len(lengths)
    stride = V + pad
    z = rs.normal(0, 3, size=(N, stride))
    z[rs.rand(N) < 0.3, rs.randint(0, V)] += 12.0
    if N > 3:
        z[2, 1:V:3] = -np.inf                      # masked vocabulary entries (the oracle admits them)
    y = rs.randint(0, V, size=N).astype(np.int32)
    if N > 3:
        y[2] = 0
    if storage == oracle.F32:
        full = z.astype(np.float32)
    elif storage == oracle.BF16:
        full = (z.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    else:
        full = z.astype(np.float64)
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    adv = np.repeat(rs.choice([1.0, -1.0, 0.0], size=R), lengths).astype(np.float64)
    seg = rs.randint(-1, 6, size=N).astype(np.int32)
    return dict(N=N, R=R, V=V, stride=stride, storage=storage, logits=full, y=y, cu=cu, adv=adv, seg=seg,
                old=rs.normal(-3, 1, size=N), use_seg=use_seg, use_old=use_old, is_mode=is_mode, gate_mode=gate_mode,
                rows=np.array(sorted(set([0, N - 1, N // 2])), np.int64), G=G,
                rewards=rs.choice([0.0, 1.0], size=R), trunc=(rs.rand(R) < 0.2).astype(np.uint8),
                K=4, seg_len=3, eps_low=0.2, eps_high=0.28, tau=0.6, sigma=4.0, denom=0.0, grad_out=-1.5)


CASES = [
    _case(1, oracle.BF16, [5, 0, 1, 9], 37, 3, False, True, oracle.IS_SAIS, oracle.GATE_PER_RESPONSE, 2),
    _case(2, oracle.F32, [1], 1, 0, True, False, oracle.IS_POIS, oracle.GATE_ALWAYS, 1),
    _case(3, oracle.F64, [7, 7, 2, 2, 30, 1], 130, 14, True, True, oracle.IS_SAIS, oracle.GATE_GLOBAL, 3),
    _case(4, oracle.BF16, [64, 3], 4099, 5, False, True, oracle.IS_SAIS, oracle.GATE_NEVER, 2),
]


@pytest.mark.parametrize("c", CASES, ids=lambda c: "N%d_V%d_st%d" % (c["N"], c["V"], c["storage"]))
def test_sanitized_oracle_matches_the_regular_build(driver, tmp_path, c):
    d = str(tmp_path)
    N, V, stride, R = c["N"], c["V"], c["stride"], c["R"]
    flat = c["logits"].reshape(-1)[:(N - 1) * stride + V]           # the last row ends at V, not at the stride
    flat.tofile(os.path.join(d, "logits.bin"))
    for name, arr in (("y.i32", c["y"]), ("cu.i32", c["cu"]), ("seg.i32", c["seg"]), ("old.f64", c["old"]),
                      ("adv.f64", c["adv"]), ("rows.i64", c["rows"]), ("rewards.f64", c["rewards"]), ("trunc.u8", c["trunc"])):
        np.ascontiguousarray(arr).tofile(os.path.join(d, name))
    rs = np.random.RandomState(N)
    B, pseg, pmax = 50, 16, 64
    prev = (rs.randint(0, 4, size=B) * pseg).astype(np.int32)
    new = np.minimum(rs.randint(1, pseg + 1, size=B), pmax - prev).astype(np.int32)
    eos = ((new < pseg) | (rs.rand(B) < 0.2)).astype(np.uint8)
    prev[0], new[0], eos[0] = 70, 99, 1                              # inconsistent sample: clamped, counted
    for name, arr in (("prev.i32", prev), ("new.i32", new), ("eos.u8", eos)):
        arr.tofile(os.path.join(d, name))
    meta = [N, V, stride, c["storage"], R, c["K"], c["seg_len"], c["is_mode"], c["gate_mode"], int(c["use_seg"]),
            int(c["use_old"]), c["eps_low"], c["eps_high"], c["tau"], c["sigma"], c["denom"], c["grad_out"],
            len(c["rows"]), c["G"], B, pseg, pmax]
    open(os.path.join(d, "meta.txt"), "w").write(" ".join(repr(x) for x in meta) + "\n")
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    proc = subprocess.run([driver, d], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert proc.returncode == 0 and "complete" in proc.stdout, proc.stdout[-4000:]

    def out(name, dtype):
        return np.fromfile(os.path.join(d, "out_" + name), dtype=dtype)

    logits = c["logits"][:, :V] if stride == V else np.lib.stride_tricks.as_strided(
        c["logits"], shape=(N, V), strides=c["logits"].strides)
    lse, logp, ent = oracle.row_stats(logits, c["y"], storage=c["storage"])
    for name, ref in (("lse.f64", lse), ("logp.f64", logp), ("ent.f64", ent)):
        np.testing.assert_array_equal(out(name, np.float64), ref, err_msg=name)
    tt = oracle.token_terms(logp, ent, c["cu"], c["adv"], c["old"] if c["use_old"] else None,
                            segment_ids=c["seg"] if c["use_seg"] else None, seg_len=c["seg_len"], eps_low=c["eps_low"],
                            eps_high=c["eps_high"], tau=c["tau"], sigma=c["sigma"], is_mode=c["is_mode"],
                            gate_mode=c["gate_mode"], denominator=c["denom"])
    assert out("loss.f64", np.float64)[0] == tt.loss
    for name, dtype, ref in (("hbar.f64", np.float64, tt.resp_entropy), ("gate.u8", np.uint8, tt.resp_gate),
                             ("seg.i32", np.int32, tt.seg), ("mask.u8", np.uint8, tt.mask), ("ratio.f64", np.float64, tt.ratio),
                             ("sur.f64", np.float64, tt.surrogate), ("g.f64", np.float64, tt.gcoef)):
        np.testing.assert_array_equal(out(name, dtype), ref, err_msg=name)
    assert out("cnt.i64", np.int64).tolist() == [tt.n_masked, tt.n_clip_inactive, tt.n_pos]
    dz = oracle.dlogits(logits, c["y"], lse, tt.gcoef, grad_out=c["grad_out"], rows=c["rows"], storage=c["storage"])
    np.testing.assert_array_equal(out("dz.f64", np.float64).reshape(dz.shape), dz)
    dg = oracle.segment_diagnostics(tt.seg, tt.ratio, logp, c["old"] if c["use_old"] else None, ent, tt.mask, c["adv"],
                                    c["K"], eps_low=c["eps_low"], eps_high=c["eps_high"])
    for name, dtype, key in (("d_count.i64", np.int64, "count"), ("d_rs.f64", np.float64, "ratio_sum"),
                             ("d_rm.f64", np.float64, "ratio_max"), ("d_clip.i64", np.int64, "clipped"),
                             ("d_kl.f64", np.float64, "kl_sum"), ("d_en.f64", np.float64, "ent_sum"),
                             ("d_mask.i64", np.int64, "masked")):
        np.testing.assert_array_equal(out(name, dtype), dg[key], err_msg=name)
    assert int(out("d_oor.i64", np.int64)[0]) == dg["out_of_range"]
    ra, keep, ta, kept = oracle.advantages(c["rewards"], c["cu"], c["G"], truncated=c["trunc"])
    np.testing.assert_array_equal(out("resp_adv.f64", np.float64), ra)
    np.testing.assert_array_equal(out("keep.u8", np.uint8), keep)
    np.testing.assert_array_equal(out("tok_adv.f64", np.float64), ta)
    assert int(out("kept.i64", np.int64)[0]) == kept
    ps = oracle.pool_step(prev, new, eos, pseg, pmax)
    for name, dtype, key in (("state.u8", np.uint8, "state"), ("total.i32", np.int32, "total_len"),
                             ("segs.i32", np.int32, "segments"), ("unf.i32", np.int32, "unfinished_idx"),
                             ("exp.i32", np.int32, "experience_idx"), ("pcu.i64", np.int64, "exp_cu_seqlens"),
                             ("ptrunc.u8", np.uint8, "exp_truncated"), ("counts.i64", np.int64, "counts")):
        np.testing.assert_array_equal(out(name, dtype), ps[key], err_msg=name)
    assert int(ps["counts"][4]) >= 1
