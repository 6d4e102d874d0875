"""Seeded sweep over shapes and settings: every case runs the two-call path and the one-call path
(both of its kernels) against the fp64 oracle, row by row.  The vocabulary sizes are drawn so that
each register shape of the row-cooperative kernel (4, 8, 15 vectors per thread), single- and
multi-piece rows, ragged last pieces and ragged last vectors all occur."""
import numpy as np
import pytest
import torch

import paper_2507_19766_amd as ulorl
import ulorl_inputs as ui
from parity import params_for, run_full_parity, sigma_between_responses

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CLUSTER_THREADS = 256


def _cases():
    rs = np.random.RandomState(20250727)
    out = []
    for i in range(40):
        dtype = "f32" if rs.rand() < 0.4 else "bf16"
        vec = 4 if dtype == "f32" else 8
        kind = i % 5
        if kind == 0:          # tiny rows: fewer elements than one vector up to a few vectors
            V = int(rs.randint(1, 6 * vec))
        elif kind == 1:        # around a multiple of one piece of a register shape (the library picks the shape from V)
            vpt = int(rs.choice([4, 8, 10, 12, 15]))
            pieces = int(rs.randint(1, 5))
            V = max(1, CLUSTER_THREADS * vpt * vec * pieces + int(rs.randint(-2 * vec, 2 * vec + 1)))
        elif kind == 2:        # small and mid-sized vocabularies
            V = int(np.exp(rs.uniform(np.log(64), np.log(40000))))
        elif kind == 3:        # large vocabularies, several pieces of 15 vectors
            V = int(np.exp(rs.uniform(np.log(40000), np.log(330000))))
        else:                  # many pieces of the smallest shape
            V = int(rs.randint(20, 60)) * CLUSTER_THREADS * 4 * vec + int(rs.randint(0, vec))
        n_resp = int(rs.randint(1, 5))
        max_len = 8 if V > 100000 else 40
        lengths = [int(rs.randint(1, max_len + 1)) for _ in range(n_resp)]
        out.append(dict(
            idx=i, dtype=dtype, V=V, lengths=lengths, seg_len=int(rs.randint(1, 17)),
            is_mode=int(rs.choice([ulorl.IS_SAIS, ulorl.IS_POIS])),
            gate=int(rs.choice([ulorl.GATE_ALWAYS, ulorl.GATE_PER_RESPONSE, ulorl.GATE_GLOBAL, ulorl.GATE_NEVER])),
            tau=float(rs.choice([0.3, 0.5, 0.9, 0.99])), eps_low=float(rs.choice([0.1, 0.2, 0.3])),
            eps_high=float(rs.choice([0.2, 0.28, 0.4])), pad=int(rs.randint(0, 4)) * vec,
            inplace=bool(rs.rand() < 0.3), forced_vpt=int(rs.choice([0, 0, 4, 8, 10, 12, 15])),
            grad_out=float(rs.choice([1.0, 1.0, -0.5, 3.0]))))
    return out


@pytest.mark.parametrize("c", _cases(), ids=lambda c: "%02d_%s_V%d_N%d" % (c["idx"], c["dtype"], c["V"], sum(c["lengths"])))
def test_random_case(c):
    base = ui.config(1) if c["dtype"] == "f32" else ui.config(2)
    w = ui.shrink(base, c["lengths"], V=c["V"], seg_len=c["seg_len"], name="sweep_%02d" % c["idx"])
    d = ui.generate(w, DEV)
    V, stride = c["V"], c["V"] + c["pad"]
    vec = 4 if c["dtype"] == "f32" else 8
    stride = (stride + vec - 1) // vec * vec            # rows stay 16-byte aligned
    buf = torch.full((w.N, stride), float("nan"), dtype=w.torch_dtype(), device=DEV)
    buf[:, :V] = d["logits"]
    d["logits"] = buf[:, :V]
    sigma = w.sigma
    if c["gate"] == ulorl.GATE_PER_RESPONSE and len(c["lengths"]) > 1:
        try:
            sigma = sigma_between_responses(ui.to_numpy_logits(d["logits"]), d["token_ids"].cpu().numpy(), w.cu_seqlens)
        except AssertionError:
            sigma = 1e9                                    # mean entropies too close together: gate every response
    elif c["gate"] == ulorl.GATE_GLOBAL:
        sigma = 1e9
    p = params_for(w, is_mode=c["is_mode"], gate_mode=c["gate"], tau=c["tau"], sigma=sigma,
                   eps_low=c["eps_low"], eps_high=c["eps_high"])
    res, tt, info = run_full_parity(w, p, data=d, inplace=c["inplace"], grad_out=c["grad_out"])
    assert int(res.counters[3]) == 0                       # no status bits
    if stride > V:
        assert torch.isnan(buf[:, V:]).all()               # padding columns are never written


def _lmhead_cases():
    rs = np.random.RandomState(20250728)
    out = []
    for i in range(16):
        hidden = 8 * int(rs.randint(1, 65)) if i % 4 else 64 * int(rs.randint(1, 9))   # K ragged or a multiple of the K tile
        V = 8 * int(rs.randint(1, 700))
        n_resp = int(rs.randint(1, 4))
        lengths = [int(rs.randint(1, 260)) for _ in range(n_resp)]
        out.append(dict(idx=i, hidden=hidden, V=V, lengths=lengths, chunk=64 * int(rs.randint(1, 40)),
                        seg_len=int(rs.randint(1, 65)), tile=int(rs.choice([7, 7, 7, 8, 6, 4, 0])),
                        is_mode=int(rs.choice([ulorl.IS_SAIS, ulorl.IS_POIS])),
                        gate=int(rs.choice([ulorl.GATE_ALWAYS, ulorl.GATE_NEVER, ulorl.GATE_GLOBAL])),
                        tau=float(rs.choice([0.02, 0.05, 0.5])), grad_out=float(rs.choice([1.0, -0.5, 2.0]))))
    # share of tokens whose advantage is set to zero (rows without a gradient, which the backward
    # pass leaves out of its products) and whether every row is kept in instead; drawn after the
    # shapes so that those stay what they were
    for c in out:
        c["dead_frac"] = float(rs.choice([0.0, 0.0, 0.3, 0.9]))
        c["dense_rows"] = bool(c["idx"] % 3 == 2)
    return out


@pytest.mark.parametrize("c", _lmhead_cases(),
                         ids=lambda c: "%02d_N%d_Hd%d_V%d_c%d_t%d" % (c["idx"], sum(c["lengths"]), c["hidden"], c["V"], c["chunk"], c["tile"]))
def test_random_lmhead_case(c):
    from parity import run_lmhead_parity
    w = ui.shrink(ui.config(5), c["lengths"], V=c["V"], hidden=c["hidden"], seg_len=c["seg_len"],
                  name="lmhead_sweep_%02d" % c["idx"])
    p = params_for(w, is_mode=c["is_mode"], gate_mode=c["gate"], tau=c["tau"],
                   sigma=1e9 if c["gate"] == ulorl.GATE_GLOBAL else w.sigma)
    launch = ulorl.Launch(gemm_tile=1 if c["tile"] == 0 else 0, gemm_group_m=c["tile"] % 5, dense_rows=c["dense_rows"])
    d = ui.generate(w, DEV)
    if c["dead_frac"] > 0.0:
        g = torch.Generator().manual_seed(1000 + c["idx"])
        dead = (torch.rand(w.N, generator=g) < c["dead_frac"]).to(DEV)
        d["advantages"] = torch.where(dead, torch.zeros_like(d["advantages"]), d["advantages"])
    res, tt = run_lmhead_parity(w, p, chunk=c["chunk"], data=d, grad_out=c["grad_out"], launch=launch)
    if c["dead_frac"] > 0.0:
        assert bool((res.gcoef[dead] == 0).all()) and bool((res.d_hidden[dead] == 0).all())
