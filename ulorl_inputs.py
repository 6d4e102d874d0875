"""Seeded synthetic inputs shaped like the paper's RL workloads.

This module serves both the GPU library's tests/benchmark and the CPU oracle's tests, and
therefore holds none of the method's arithmetic: it only draws random tensors.  Where a
recipe needs "the current log-prob" to build the behaviour-policy log-prob (old = current +
noise), it calls the framework's stock ``log_softmax`` -- the result is just another input
that both sides consume.

Shapes follow the training set-up of Sec. 4.1 (responses of up to 128k tokens cut into 16k
segments, binary rewards hence advantages of either sign, tau = 0.99) with a Qwen3-sized
vocabulary of 151 936 and hidden size 2048.  The private RL data set and the trained policy
are replaced by Gaussian logits with a fraction of "peaked" rows, so that some sampled
tokens exceed the MPT probability threshold.

Generation is blocked by ``ROWS_PER_BLOCK`` rows with one counter-based seed per block, so a
row's values do not depend on how many rows are generated, and tensors larger than host or
device scratch memory can be produced block by block.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Callable, Dict, Optional

import numpy as np
import torch

ROWS_PER_BLOCK = 256


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    lengths: tuple            # tokens per response
    V: int
    dtype: str                # "f32" | "bf16"  (storage type of the logits)
    seg_len: int              # segment length; segment id = offset_in_response // seg_len
    logit_std: float
    spike_frac: float         # fraction of rows with one boosted logit
    spike_boost: float
    old_noise_std: float      # std of (old_logp - current logp) ...
    old_noise_per_segment: bool = False   # ... multiplied by the segment index if True
    advantages: tuple = ()    # one value per response
    eps_low: float = 0.2
    eps_high: float = 0.2
    tau: float = 0.99
    sigma: float = 0.2
    hidden: int = 0           # >0: lm_head variant, logits = hidden_states @ weight
    weight_std: float = 0.02
    # lm_head variant only: this fraction of the hidden rows is replaced by a multiple of one column
    # of the weight, scaled so that the column's logit stands ln(V) + U(align_margin) above zero:
    # such rows are "peaked" (probability of that token from ~0.9 to ~1), so some sampled tokens
    # exceed the MPT threshold.  0 leaves the recipe (and its random streams) unchanged.
    align_frac: float = 0.0
    align_margin: tuple = (2.5, 9.0)

    @property
    def R(self) -> int:
        return len(self.lengths)

    @property
    def N(self) -> int:
        return int(sum(self.lengths))

    @property
    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.lengths)]).astype(np.int32)

    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


def _log_uniform_lengths(seed: int, count: int, lo: int, hi: int) -> tuple:
    rs = np.random.RandomState(seed)
    u = rs.uniform(math.log(lo), math.log(hi), size=count)
    return tuple(int(x) for x in np.floor(np.exp(u)))


def config(index: int) -> Workload:
    """The five workload configurations, 1-based."""
    if index == 1:   # tiny, CPU-checkable, fp32
        return Workload("cfg1_tiny_f32", 1001, (1024, 1024), 4096, "f32", 512, 2.0, 0.20, 12.0,
                        0.05, advantages=(1.0, -1.0))
    if index == 2:   # Qwen3-sized vocabulary, short outputs
        return Workload("cfg2_8x8192_bf16", 1002, (8192,) * 8, 151936, "bf16", 4096, 3.0, 0.30,
                        15.0, 0.1, advantages=(1.0, -1.0) * 4)
    if index == 3:   # long-tail variable-length batch, packed
        lengths = _log_uniform_lengths(1003, 16, 1024, 65536)
        adv = tuple(1.0 if i % 2 == 0 else -1.0 for i in range(16))
        return Workload("cfg3_varlen_bf16", 1003, lengths, 151936, "bf16", 16384, 3.0, 0.30,
                        15.0, 0.1, advantages=adv)
    if index == 4:   # one ultra-long output, 8 segments with growing staleness
        return Workload("cfg4_1x131072_bf16", 1004, (131072,), 151936, "bf16", 16384, 3.0, 0.40,
                        15.0, 0.02, old_noise_per_segment=True, advantages=(1.0,))
    if index == 5:   # lm_head variant: logits are never materialised by the library
        return Workload("cfg5_lmhead_bf16", 1005, (16384, 16384), 151936, "bf16", 8192, 0.0,
                        0.0, 0.0, 0.1, advantages=(1.0, -1.0), hidden=2048, weight_std=0.02)
    raise ValueError("config index must be 1..5")


def shrink(w: Workload, lengths, V: Optional[int] = None, seg_len: Optional[int] = None,
           hidden: Optional[int] = None, name: Optional[str] = None) -> Workload:
    """Same recipe at a reduced size (for oracle-sized parity cases)."""
    lengths = tuple(int(x) for x in lengths)
    adv = tuple(w.advantages[i % len(w.advantages)] for i in range(len(lengths)))
    return replace(w, lengths=lengths, V=V or w.V, seg_len=seg_len or w.seg_len,
                   hidden=(hidden if hidden is not None else w.hidden), advantages=adv,
                   name=name or (w.name + "_small"))


def _block_generator(w: Workload, block: int, device, stream: int = 0) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((w.seed * 1_000_003 + block) * 8 + stream)
    return g


def _response_of_rows(w: Workload) -> np.ndarray:
    return np.repeat(np.arange(w.R, dtype=np.int64), np.asarray(w.lengths, dtype=np.int64))


def per_token_metadata(w: Workload) -> Dict[str, np.ndarray]:
    """Host-side integer/broadcast metadata: response index, segment id, advantage per token."""
    resp = _response_of_rows(w)
    cu = w.cu_seqlens.astype(np.int64)
    offs = np.arange(w.N, dtype=np.int64) - cu[resp]
    seg = (offs // w.seg_len).astype(np.int32)
    adv = np.asarray(w.advantages, dtype=np.float32)[resp]
    return {"response": resp.astype(np.int32), "segment_ids": seg, "advantages": adv}


def _sample_tokens(z_f32: torch.Tensor, gen: torch.Generator) -> torch.Tensor:
    """y ~ Categorical(softmax(z)) by the Gumbel-max construction (argmax of z + Gumbel noise)."""
    u = torch.rand(z_f32.shape, generator=gen, device=z_f32.device, dtype=torch.float32)
    u.clamp_(min=1e-20, max=1.0 - 1e-7)
    gumbel = -torch.log(-torch.log(u))
    return torch.argmax(z_f32 + gumbel, dim=-1).to(torch.int32)


def _behaviour_logp(z_f32: torch.Tensor, y: torch.Tensor) -> torch.Tensor:
    """Centre of the recorded behaviour-policy log-probs of a block: the framework's stock fp32
    log_softmax at the sampled tokens.  INPUT GENERATION ONLY -- the result (plus noise) is handed to
    both sides as ``old_logp``; neither the library nor the oracle computes anything through it."""
    return torch.log_softmax(z_f32, dim=-1).gather(1, y.long().unsqueeze(1)).squeeze(1)


def generate(w: Workload, device="cpu", logits_out: Optional[torch.Tensor] = None,
             progress: Optional[Callable[[int, int], None]] = None) -> Dict[str, torch.Tensor]:
    """Materialise one workload on ``device``.

    Returns a dict with ``logits`` [N, V] (storage dtype of the workload; for the lm_head
    variant instead ``hidden`` [N, Hd] and ``weight`` [Hd, V], both bf16), ``token_ids`` int32
    [N], ``old_logp`` fp32 [N], ``advantages`` fp32 [N], ``segment_ids`` int32 [N],
    ``cu_seqlens`` int32 [R+1].
    """
    device = torch.device(device)
    meta = per_token_metadata(w)
    seg_t = torch.from_numpy(meta["segment_ids"]).to(device)
    out: Dict[str, torch.Tensor] = {
        "cu_seqlens": torch.from_numpy(w.cu_seqlens).to(device),
        "segment_ids": seg_t,
        "advantages": torch.from_numpy(meta["advantages"]).to(device),
    }
    N, V = w.N, w.V
    token_ids = torch.empty(N, dtype=torch.int32, device=device)
    old_logp = torch.empty(N, dtype=torch.float32, device=device)

    if w.hidden > 0:
        gw = _block_generator(w, 0, device, stream=7)
        weight = (torch.randn(w.hidden, V, generator=gw, device=device, dtype=torch.float32)
                  * w.weight_std).to(torch.bfloat16)
        hidden = torch.empty(N, w.hidden, dtype=torch.bfloat16, device=device)
        wf = weight.float()
    else:
        logits = logits_out if logits_out is not None else torch.empty(
            N, V, dtype=w.torch_dtype(), device=device)
        assert logits.shape == (N, V) and logits.dtype == w.torch_dtype()

    n_blocks = (N + ROWS_PER_BLOCK - 1) // ROWS_PER_BLOCK
    for b in range(n_blocks):
        r0 = b * ROWS_PER_BLOCK
        r1 = min(N, r0 + ROWS_PER_BLOCK)
        rows = r1 - r0
        g = _block_generator(w, b, device)
        if w.hidden > 0:
            h = torch.randn(ROWS_PER_BLOCK, w.hidden, generator=g, device=device,
                            dtype=torch.float32)[:rows].to(torch.bfloat16)
            if w.align_frac > 0.0:
                aligned = torch.rand(ROWS_PER_BLOCK, generator=g, device=device)[:rows] < w.align_frac
                col = torch.randint(0, V, (ROWS_PER_BLOCK,), generator=g, device=device)[:rows]
                lo, hi = w.align_margin
                margin = lo + (hi - lo) * torch.rand(ROWS_PER_BLOCK, generator=g, device=device)[:rows]
                wc = wf[:, col]                                   # [Hd, rows]
                scale = (math.log(V) + margin) / (wc * wc).sum(0)
                h = torch.where(aligned[:, None], (wc * scale).t().to(torch.bfloat16), h)
            hidden[r0:r1] = h
            zf = h.float() @ wf                      # stock GEMM: only used to draw y and old_logp
        else:
            z = torch.randn(ROWS_PER_BLOCK, V, generator=g, device=device,
                            dtype=torch.float32)[:rows] * w.logit_std
            spiked = torch.rand(ROWS_PER_BLOCK, generator=g, device=device)[:rows] < w.spike_frac
            where = torch.randint(0, V, (ROWS_PER_BLOCK,), generator=g, device=device)[:rows]
            ridx = torch.arange(rows, device=device)
            z[ridx, where] += spiked.to(torch.float32) * w.spike_boost
            # rounded to the storage type by an elementwise kernel writing in place (fp32 source: a
            # converting copy; no staging tensor, no device-to-device memcpy of the block)
            torch.mul(z, 1.0, out=logits[r0:r1])
            zf = logits[r0:r1].float()
        y = _sample_tokens(zf, g)
        cur = _behaviour_logp(zf, y)
        noise = torch.randn(ROWS_PER_BLOCK, generator=g, device=device, dtype=torch.float32)[:rows]
        scale = torch.full((rows,), w.old_noise_std, device=device, dtype=torch.float32)
        if w.old_noise_per_segment:
            scale = scale * seg_t[r0:r1].to(torch.float32)
        token_ids[r0:r1] = y
        old_logp[r0:r1] = cur + scale * noise
        if progress is not None:
            progress(b + 1, n_blocks)

    out["token_ids"] = token_ids
    out["old_logp"] = old_logp
    if w.hidden > 0:
        out["hidden"] = hidden
        out["weight"] = weight
    else:
        out["logits"] = logits
    return out


def to_numpy_logits(t: torch.Tensor) -> np.ndarray:
    """Host view of a logits tensor for the oracle: fp32 stays fp32, bf16 becomes raw uint16."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
