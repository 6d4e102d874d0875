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
