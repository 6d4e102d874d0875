"""Test harness: training with segment rollouts (Algorithm 1, Sec. 3.1.1) on synthetic response
lengths, driving a pool update passed in as a callable (the oracle's, or the GPU entry point's).
It belongs to neither side: it holds the loop and a cost model, none of the pool update's logic.

The loop is the paper's: every step decodes at most one segment for each sample in flight
(samples carried over from the unfinished pool first, then new prompts up to the rollout batch
size), sorts the samples into the unfinished and the experience pool with
``ulorl_segment_pool_step``, and trains on the experience pool.  What a step costs is a MODEL, not
a measurement: decoding lasts as long as the longest decode of the step (every sample waits for
it), the rest is a constant plus, optionally, a share proportional to the tokens trained on.  The
default constants are solved from the first two rows of the paper's Table 1 (64k outputs: 1240 s
and 774 s per step with one and two segments); the model is there to show the trend and to
exercise the pool bookkeeping over many steps, not to predict wall-clock.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List

import numpy as np


@dataclass
class StepCost:
    """Seconds = fixed + per_decoded_token * (longest decode of the step) + per_trained_token * tokens.
    The defaults solve  fixed + 65536 d = 1240  and  fixed + 32768 d = 774  (Table 1, one and two
    segments of a 64k output); the table's third row (four segments, 601 s) is then predicted as
    541 s.  A training share can be split off the fixed part with per_trained_token."""
    fixed: float = 308.0
    per_decoded_token: float = 932.0 / 65536.0
    per_trained_token: float = 0.0


def synthetic_lengths(n: int, max_len: int, seed: int, median_frac: float = 0.22, sigma: float = 0.9) -> np.ndarray:
    """Long-tailed response lengths (log-normal, median = median_frac * max_len): most samples end
    well inside max_len, a few would run past it (those get truncated there)."""
    rng = np.random.default_rng(seed)
    x = rng.lognormal(mean=np.log(median_frac * max_len), sigma=sigma, size=n)
    return np.maximum(1, np.floor(x)).astype(np.int64)


def simulate(pool_step: Callable, full_len: np.ndarray, *, batch: int, segments: int, max_len: int, steps: int,
             cost: StepCost = StepCost()) -> Dict[str, object]:
    """Runs `steps` rollout steps over the prompt stream whose latent response lengths are
    `full_len` (consumed in order).  `pool_step(prev_len, new_len, hit_eos, seg_len, max_len)` is
    the pool update (the GPU entry point or a reference of it) returning a dict of numpy arrays.
    Returns per-step records and totals."""
    assert max_len % segments == 0
    seg_len = max_len // segments
    next_prompt = 0
    carried_len = np.zeros(0, np.int64)       # latent length of the samples in the unfinished pool
    carried_prev = np.zeros(0, np.int64)      # tokens they have decoded so far
    carried_id = np.zeros(0, np.int64)
    done: List[tuple] = []                    # (prompt id, trained length, truncated)
    records = []
    total_time = 0.0
    for _ in range(steps):
        fresh = min(batch - carried_len.shape[0], full_len.shape[0] - next_prompt)
        ids = np.concatenate([carried_id, np.arange(next_prompt, next_prompt + fresh)])
        lat = np.concatenate([carried_len, full_len[next_prompt:next_prompt + fresh]])
        prev = np.concatenate([carried_prev, np.zeros(fresh, np.int64)])
        next_prompt += fresh
        if ids.shape[0] == 0:
            break
        new = np.minimum(np.minimum(seg_len, lat - prev), max_len - prev)
        eos = (prev + new == lat) & (lat <= max_len)
        out = pool_step(prev.astype(np.int32), new.astype(np.int32), eos.astype(np.uint8), seg_len, max_len)
        unf = np.asarray(out["unfinished_idx"], np.int64)
        exp = np.asarray(out["experience_idx"], np.int64)
        cu = np.asarray(out["exp_cu_seqlens"], np.int64)
        trunc = np.asarray(out["exp_truncated"], np.uint8)
        for k, i in enumerate(exp):
            done.append((int(ids[i]), int(cu[k + 1] - cu[k]), int(trunc[k])))
        tokens = int(cu[-1]) if cu.shape[0] else 0
        t = cost.fixed + cost.per_decoded_token * float(new.max()) + cost.per_trained_token * tokens
        total_time += t
        records.append({"in_flight": int(ids.shape[0]), "fresh": int(fresh), "finished": int(exp.shape[0]),
                        "unfinished": int(unf.shape[0]), "tokens": tokens, "longest_decode": int(new.max()),
                        "seconds": t, "inconsistent": int(np.asarray(out["counts"])[4])})
        carried_id, carried_len = ids[unf], lat[unf]
        carried_prev = np.asarray(out["total_len"], np.int64)[unf]
    n_steps = len(records)
    trained_tokens = sum(r["tokens"] for r in records)
    return {"records": records, "done": done, "steps": n_steps, "seconds": total_time,
            "seconds_per_step": total_time / max(n_steps, 1), "trained_samples": len(done),
            "trained_tokens": trained_tokens, "tokens_per_second": trained_tokens / max(total_time, 1e-30),
            "left_unfinished": int(carried_id.shape[0])}


def gpu_pool_step(prev_len, new_len, hit_eos, seg_len, max_len):
    """`pool_step` callable backed by ulorl_segment_pool_step (numpy in, numpy out, trimmed to the counts)."""
    import torch

    import paper_2507_19766_amd as ulorl

    dev = torch.device("cuda:0")
    out = ulorl.segment_pool_step(torch.from_numpy(np.ascontiguousarray(prev_len)).to(dev),
                                    torch.from_numpy(np.ascontiguousarray(new_len)).to(dev),
                                    torch.from_numpy(np.ascontiguousarray(hit_eos)).to(dev), seg_len, max_len)
    host = {k: v.cpu().numpy() for k, v in out.items()}
    nu, ne = int(host["counts"][0]), int(host["counts"][1])
    host["unfinished_idx"] = host["unfinished_idx"][:nu]
    host["experience_idx"] = host["experience_idx"][:ne]
    host["exp_cu_seqlens"] = host["exp_cu_seqlens"][:ne + 1]
    host["exp_truncated"] = host["exp_truncated"][:ne]
    return host
