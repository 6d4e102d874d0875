"""Host-side checks of the seeded synthetic-input recipes (shapes, determinism, structure)."""
import numpy as np
import torch

import ulorl_inputs as ui


def test_config_shapes_follow_the_paper_geometry():
    c1, c2, c3, c4, c5 = (ui.config(i) for i in range(1, 6))
    assert (c1.N, c1.V, c1.dtype, c1.seg_len) == (2048, 4096, "f32", 512)
    assert (c2.R, c2.N, c2.V, c2.seg_len) == (8, 65536, 151936, 4096)
    assert c3.R == 16 and all(1024 <= L <= 65536 for L in c3.lengths)
    assert c3.N * c3.V * 2 < 200e9             # packed logits must fit beside their gradient
    # one 128k-token response in 8 segments of 16k (Sec. 4.1)
    assert (c4.R, c4.N, c4.seg_len, c4.N // c4.seg_len) == (1, 131072, 16384, 8)
    assert (c5.N, c5.hidden, c5.V) == (32768, 2048, 151936)
    for c in (c1, c2, c3, c4, c5):
        assert (c.tau, c.sigma) == (0.99, 0.2)   # Sec. 4.1
        cu = c.cu_seqlens
        assert cu[0] == 0 and cu[-1] == c.N and np.all(np.diff(cu) > 0)


def test_generation_is_deterministic_and_block_independent():
    w = ui.shrink(ui.config(2), [300, 17, 400], V=1000, seg_len=128)
    a = ui.generate(w)
    b = ui.generate(w)
    for k in a:
        assert torch.equal(a[k], b[k]), k
    # the first rows do not depend on how many rows follow
    w2 = ui.shrink(ui.config(2), [300], V=1000, seg_len=128)
    c = ui.generate(w2)
    assert torch.equal(c["logits"][:256], a["logits"][:256])
    assert torch.equal(c["token_ids"][:256], a["token_ids"][:256])
    assert a["logits"].dtype == torch.bfloat16 and a["token_ids"].dtype == torch.int32
    assert int(a["token_ids"].min()) >= 0 and int(a["token_ids"].max()) < 1000


def test_metadata_and_value_structure():
    w = ui.shrink(ui.config(4), [700], V=2048, seg_len=100)
    d = ui.generate(w)
    seg = d["segment_ids"].numpy()
    np.testing.assert_array_equal(seg, np.arange(700) // 100)
    z = d["logits"].float()
    cur = torch.log_softmax(z, -1).gather(1, d["token_ids"].long()[:, None])[:, 0]
    diff = (d["old_logp"] - cur).numpy()
    assert np.all(diff[seg == 0] == 0.0)                  # first segment exactly on-policy
    for k in (1, 3, 6):
        assert 0.3 * 0.02 * k < diff[seg == k].std() < 3 * 0.02 * k
    assert torch.all(d["advantages"] == 1.0)
    # roughly 40 % of rows carry a +15 spike
    frac = float(((z.max(1).values - z.median(1).values) > 12).float().mean())
    assert 0.3 < frac < 0.5


def test_tiny_config_has_tokens_above_the_mpt_threshold():
    d = ui.generate(ui.config(1))
    z = d["logits"].double()
    p = torch.softmax(z, -1).gather(1, d["token_ids"].long()[:, None])[:, 0]
    assert d["logits"].dtype == torch.float32
    assert 5 <= int((p >= 0.99).sum()) <= 200
    adv = d["advantages"].numpy()
    assert np.all(adv[:1024] == 1.0) and np.all(adv[1024:] == -1.0)


def test_lm_head_variant_inputs():
    w = ui.shrink(ui.config(5), [40, 24], V=512, hidden=64, seg_len=16)
    d = ui.generate(w)
    assert d["hidden"].shape == (64, 64) and d["weight"].shape == (64, 512)
    assert d["hidden"].dtype == torch.bfloat16 and d["weight"].dtype == torch.bfloat16
    assert "logits" not in d
    assert abs(float(d["weight"].float().std()) - 0.02) < 0.002
