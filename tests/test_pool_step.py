"""Pins of the oracle's segment-rollout pool update (Algorithm 1, Sec. 3.1.1) and of the
rollout model built on it.  CPU only."""
import os

import numpy as np
import pytest

import oracle
import rollout_sim as rm

HERE = os.path.dirname(os.path.abspath(__file__))


def test_three_ways_a_decode_ends_by_hand():
    # seg_len 16, max_len 64
    #  0: new prompt, segment full, no end token             -> unfinished, 16 tokens, 1 segment
    #  1: 16 + 5, end token                                   -> finished, 21 tokens, 2 segments
    #  2: new prompt, end token after 7                       -> finished
    #  3: 48 + 16 = 64 = max_len, no end token                -> truncated, 4 segments
    #  4: 48 + 16 = 64 with the end token exactly at the limit -> finished, not truncated
    #  5: 60 + 4 = 64: the limit cuts the segment short        -> truncated
    #  6: 32 + 16 = 48 < 64, segment full                      -> unfinished, 3 segments
    r = oracle.pool_step([0, 16, 0, 48, 48, 60, 32], [16, 5, 7, 16, 16, 4, 16], [0, 1, 1, 0, 1, 0, 0], 16, 64)
    assert r["state"].tolist() == [0, 1, 1, 2, 1, 2, 0]
    assert r["total_len"].tolist() == [16, 21, 7, 64, 64, 64, 48]
    assert r["segments"].tolist() == [1, 2, 1, 4, 4, 4, 3]
    assert r["unfinished_idx"].tolist() == [0, 6]
    assert r["experience_idx"].tolist() == [1, 2, 3, 4, 5]
    assert r["exp_cu_seqlens"].tolist() == [0, 21, 28, 92, 156, 220]
    assert r["exp_truncated"].tolist() == [0, 0, 1, 0, 1]
    assert r["counts"].tolist() == [2, 5, 2, 220, 0]


def test_inconsistent_samples_are_counted_and_kept_unfinished():
    # stopped early without a reason; more tokens than the segment holds; more than max_len allows;
    # an end flag without a token; a sample that was already at the limit
    r = oracle.pool_step([0, 0, 60, 16, 64], [5, 17, 9, 0, 0], [0, 0, 0, 1, 0], 16, 64)
    assert r["counts"][4] == 5
    assert r["state"].tolist() == [0, 0, 0, 0, 0]
    assert r["unfinished_idx"].tolist() == [0, 1, 2, 3, 4]
    assert (r["total_len"] <= 64).all() and (r["total_len"] >= 0).all()
    with pytest.raises(ValueError):
        oracle.pool_step([0], [1], [0], 0, 64)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_partition_invariants_on_random_steps(seed):
    rng = np.random.default_rng(seed)
    B, seg, mx = 3000, 64, 640
    prev = rng.integers(0, mx // seg, B) * seg
    room = np.minimum(seg, mx - prev)
    kind = rng.integers(0, 3, B)                      # 0: fills the segment, 1: ends early with the end token, 2: ends at the fill point
    new = np.where(kind == 1, rng.integers(1, room + 1), room)
    eos = (kind >= 1).astype(np.uint8)
    r = oracle.pool_step(prev, new, eos, seg, mx)
    assert r["counts"][4] == 0
    unf, exp = r["unfinished_idx"], r["experience_idx"]
    assert sorted(np.concatenate([unf, exp]).tolist()) == list(range(B))      # every sample in exactly one pool
    assert (np.diff(unf) > 0).all() and (np.diff(exp) > 0).all()             # order preserved
    tot = prev + new
    assert (r["total_len"] == tot).all()
    assert (r["exp_cu_seqlens"] == np.concatenate([[0], np.cumsum(tot[exp])])).all()
    assert (r["state"][unf] == 0).all() and (r["state"][exp] > 0).all()
    assert ((r["state"] == 1) == (eos != 0)).all()
    assert ((r["state"] == 2) == ((eos == 0) & (tot >= mx))).all()
    assert (r["exp_truncated"] == (r["state"][exp] == 2)).all()
    assert r["counts"].tolist()[:4] == [len(unf), len(exp), int((r["state"] == 2).sum()), int(tot[exp].sum())]
    assert (tot[unf] % seg == 0).all() and (tot[unf] < mx).all()             # unfinished samples sit on a segment boundary


def test_one_segment_is_plain_rollout():
    L = rm.synthetic_lengths(4000, 4096, 3)
    r = rm.simulate(oracle.pool_step, L, batch=100, segments=1, max_len=4096, steps=40)
    assert all(rec["unfinished"] == 0 and rec["finished"] == 100 for rec in r["records"])


@pytest.mark.parametrize("segments", [2, 4, 8])
def test_every_prompt_is_trained_exactly_once_with_its_own_length(segments):
    """Conservation over a whole run: the pools lose and duplicate nothing, a sample's trained
    length is its latent length cut at max_len, and it is marked truncated iff it was cut."""
    mx = 4096
    L = rm.synthetic_lengths(3000, mx, 11)
    r = rm.simulate(oracle.pool_step, L, batch=64, segments=segments, max_len=mx, steps=10_000)
    assert all(rec["inconsistent"] == 0 for rec in r["records"])
    assert r["left_unfinished"] == 0 and r["trained_samples"] == 3000
    ids = [d[0] for d in r["done"]]
    assert sorted(ids) == list(range(3000))
    for pid, length, trunc in r["done"]:
        assert length == min(int(L[pid]), mx)
        assert trunc == int(L[pid] > mx)
    # no step decodes more than one segment per sample
    assert max(rec["longest_decode"] for rec in r["records"]) <= mx // segments


def test_step_time_follows_the_trend_of_table_1():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "table1_segment_speed.txt")) if l[0] != "#"]
    paper = {int(s): (float(t), float(x)) for s, t, x in rows}
    L = rm.synthetic_lengths(200_000, 65536, 7)
    sec = {s: rm.simulate(oracle.pool_step, L, batch=128, segments=s, max_len=65536, steps=300)["seconds_per_step"]
           for s in (1, 2, 4, 8)}
    assert sec[1] > sec[2] > sec[4] > sec[8]                                   # more segments, shorter steps ...
    assert sec[1] / sec[8] < 8 and sec[1] / sec[4] < 4                         # ... but less than proportionally
    # the cost constants are solved from the first two printed rows; the third is a prediction
    assert abs(sec[1] - paper[1][0]) < 1 and abs(sec[2] - paper[2][0]) < 1
    assert abs(sec[4] - paper[4][0]) / paper[4][0] < 0.12
    assert abs(sec[1] / sec[2] - paper[2][1]) < 0.01
