"""ctypes front end of the fp64 CPU oracle (``ulorl_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the benchmark's
reported CPU baseline.  It neither imports nor is imported by the GPU package.  Apart from
argument marshalling for the C functions its only arithmetic is the lm_head variant's three
stock fp64 matrix products (numpy), which are that variant's definition.

The three main C entry points mirror the three stages of the objective of Sec. 3.2.2:
row statistics over the vocabulary, the O(1)-per-token terms, and the logits gradient; three
more cover the pool update of the segment-rollout loop (Algorithm 1), the group advantages of
Eq. 4 / Eq. 7 / Sec. 3.5 and per-segment diagnostics (Sec. 3.1.2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ulorl_oracle.c")
_LIB = os.path.join(_HERE, "_build", "libulorl_oracle.so")

F32, BF16, F64 = 0, 1, 2
IS_SAIS, IS_POIS = 0, 1
GATE_PER_RESPONSE, GATE_GLOBAL, GATE_ALWAYS, GATE_NEVER = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-fPIC", "-shared",
             _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("ulorl_oracle_row_stats", "ulorl_oracle_token_terms",
                     "ulorl_oracle_dlogits", "ulorl_oracle_threads"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _storage(logits: np.ndarray, storage):
    if storage is not None:
        return storage
    if logits.dtype == np.float32:
        return F32
    if logits.dtype == np.float64:
        return F64
    if logits.dtype == np.uint16:
        return BF16
    raise TypeError("logits must be float32, float64 or uint16 (raw bfloat16)")


def threads() -> int:
    return int(_load().ulorl_oracle_threads())


def row_stats(logits: np.ndarray, token_ids: np.ndarray, storage=None):
    """-> (lse, logp, entropy), float64 [N].  ``logits`` is [N, V] C-contiguous rows
    (row stride = logits.strides[0]); uint16 means raw bfloat16."""
    assert logits.ndim == 2 and logits.strides[1] == logits.itemsize
    st = _storage(logits, storage)
    n, v = logits.shape
    stride = logits.strides[0] // logits.itemsize
    y = np.ascontiguousarray(token_ids, dtype=np.int32)
    lse = np.empty(n, np.float64)
    logp = np.empty(n, np.float64)
    ent = np.empty(n, np.float64)
    rc = _load().ulorl_oracle_row_stats(
        _ptr(logits), ctypes.c_int(st), ctypes.c_int64(n), ctypes.c_int64(v),
        ctypes.c_int64(stride), _ptr(y), _ptr(lse), _ptr(logp), _ptr(ent))
    if rc != 0:
        raise ValueError("oracle row_stats: token id out of range")
    return lse, logp, ent


@dataclass
class TokenTerms:
    loss: float
    resp_entropy: np.ndarray
    resp_gate: np.ndarray
    seg: np.ndarray
    mask: np.ndarray
    ratio: np.ndarray
    surrogate: np.ndarray
    gcoef: np.ndarray
    n_masked: int
    n_clip_inactive: int
    n_pos: int


def token_terms(logp, entropy, cu_seqlens, advantages, old_logp=None, *, segment_ids=None,
                seg_len=0, eps_low=0.2, eps_high=0.2, tau=0.99, sigma=0.2, is_mode=IS_SAIS,
                gate_mode=GATE_PER_RESPONSE, denominator=0.0) -> TokenTerms:
    logp = np.ascontiguousarray(logp, np.float64)
    ent = np.ascontiguousarray(entropy, np.float64)
    n = logp.shape[0]
    cu = np.ascontiguousarray(cu_seqlens, np.int32)
    r = cu.shape[0] - 1
    adv = np.ascontiguousarray(advantages, np.float64)
    if old_logp is None:
        if is_mode != IS_POIS:
            raise ValueError("old_logp may be omitted only in POIS mode")
        old = None
    else:
        old = np.ascontiguousarray(old_logp, np.float64)
    segs = None if segment_ids is None else np.ascontiguousarray(segment_ids, np.int32)
    loss = ctypes.c_double(0.0)
    hbar = np.empty(r, np.float64)
    gate = np.empty(r, np.uint8)
    seg = np.empty(n, np.int32)
    mask = np.empty(n, np.uint8)
    ratio = np.empty(n, np.float64)
    sur = np.empty(n, np.float64)
    g = np.empty(n, np.float64)
    cnt = np.zeros(3, np.int64)
    rc = _load().ulorl_oracle_token_terms(
        ctypes.c_int64(n), _ptr(logp), _ptr(ent), _ptr(cu), ctypes.c_int32(r), _ptr(segs),
        ctypes.c_int32(seg_len), _ptr(old), _ptr(adv), ctypes.c_double(eps_low),
        ctypes.c_double(eps_high), ctypes.c_double(tau), ctypes.c_double(sigma),
        ctypes.c_int(is_mode), ctypes.c_int(gate_mode), ctypes.c_double(denominator),
        ctypes.byref(loss), _ptr(hbar), _ptr(gate), _ptr(seg), _ptr(mask), _ptr(ratio),
        _ptr(sur), _ptr(g), _ptr(cnt))
    if rc != 0:
        raise ValueError("oracle token_terms: malformed cu_seqlens (rc=%d)" % rc)
    return TokenTerms(loss.value, hbar, gate, seg, mask, ratio, sur, g,
                      int(cnt[0]), int(cnt[1]), int(cnt[2]))


def dlogits(logits: np.ndarray, token_ids, lse, gcoef, grad_out=1.0, rows=None, storage=None):
    """-> float64 [len(rows) or N, V]: grad_out * g_t * (onehot(y_t) - softmax(z_t))."""
    assert logits.ndim == 2 and logits.strides[1] == logits.itemsize
    st = _storage(logits, storage)
    n, v = logits.shape
    stride = logits.strides[0] // logits.itemsize
    y = np.ascontiguousarray(token_ids, dtype=np.int32)
    lse = np.ascontiguousarray(lse, np.float64)
    g = np.ascontiguousarray(gcoef, np.float64)
    if rows is None:
        sel, nsel = None, n
    else:
        sel = np.ascontiguousarray(rows, np.int64)
        nsel = sel.shape[0]
    out = np.empty((nsel, v), np.float64)
    _load().ulorl_oracle_dlogits(
        _ptr(logits), ctypes.c_int(st), ctypes.c_int64(v), ctypes.c_int64(stride), _ptr(y),
        _ptr(lse), _ptr(g), ctypes.c_double(grad_out), _ptr(sel), ctypes.c_int64(nsel),
        _ptr(out))
    return out


# ------------------------------------------------------------------------------------ lm_head variant
# The variant's definition is "the same objective with logits = hidden . W": the oracle forms the
# logits with a stock fp64 matrix product and feeds them to the functions above; the two weight
# gradients are the chain rule through that product.

def bf16_to_f64(raw: np.ndarray) -> np.ndarray:
    """Exact decode of raw bfloat16 (uint16) to float64."""
    return (raw.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def lmhead_logits(hidden_raw: np.ndarray, weight_raw: np.ndarray) -> np.ndarray:
    """z = hidden [N, Hd] . W [Hd, V] in fp64 from raw-bf16 operands."""
    return bf16_to_f64(hidden_raw) @ bf16_to_f64(weight_raw)


def lmhead_grads(hidden_raw: np.ndarray, weight_raw: np.ndarray, dz: np.ndarray):
    """d_hidden = dz . W^T  [N, Hd],  d_W = hidden^T . dz  [Hd, V]   (fp64)."""
    h = bf16_to_f64(hidden_raw)
    w = bf16_to_f64(weight_raw)
    return dz @ w.T, h.T @ dz


# ------------------------------------------------------------------------------------ neighbours of the hot path

def advantages(rewards, cu_seqlens, group_size, truncated=None, eps=1e-6, unbiased=False):
    """Group-relative advantages with the dynamic-sampling filter and overlong punishment.
    -> (resp_adv [R], group_keep [R/G], token_adv [N], kept_tokens)."""
    rew = np.ascontiguousarray(rewards, np.float64)
    R = rew.shape[0]
    cu = np.ascontiguousarray(cu_seqlens, np.int32)
    N = int(cu[-1])
    tr = None if truncated is None else np.ascontiguousarray(truncated, np.uint8)
    resp = np.empty(R, np.float64)
    keep = np.empty(max(R // max(group_size, 1), 1), np.uint8)
    tok = np.empty(N, np.float64)
    kept = ctypes.c_int64(0)
    lib = _load()
    lib.ulorl_oracle_advantages.restype = ctypes.c_int
    rc = lib.ulorl_oracle_advantages(
        ctypes.c_int32(R), ctypes.c_int32(group_size), _ptr(rew), _ptr(tr), _ptr(cu), ctypes.c_int64(N),
        ctypes.c_double(eps), ctypes.c_int(1 if unbiased else 0), _ptr(resp), _ptr(keep), _ptr(tok),
        ctypes.byref(kept))
    if rc != 0:
        raise ValueError("oracle advantages: rc=%d" % rc)
    return resp, keep[:R // group_size], tok, int(kept.value)


def segment_diagnostics(seg, ratio, logp, old_logp, entropy, mask, advantages, K, eps_low=0.2, eps_high=0.2):
    """-> dict of per-segment arrays (count, ratio_sum, ratio_max, clipped, kl_sum, ent_sum, masked)
    and the number of tokens with a segment id outside [0, K)."""
    seg = np.ascontiguousarray(seg, np.int32)
    N = seg.shape[0]
    f = lambda a: None if a is None else np.ascontiguousarray(a, np.float64)
    ratio, logp, old_logp, entropy, adv = f(ratio), f(logp), f(old_logp), f(entropy), f(advantages)
    mask = np.ascontiguousarray(mask, np.uint8)
    out = {"count": np.zeros(K, np.int64), "ratio_sum": np.zeros(K), "ratio_max": np.zeros(K),
           "clipped": np.zeros(K, np.int64), "kl_sum": np.zeros(K), "ent_sum": np.zeros(K),
           "masked": np.zeros(K, np.int64)}
    oor = ctypes.c_int64(0)
    lib = _load()
    lib.ulorl_oracle_segment_diagnostics.restype = ctypes.c_int
    lib.ulorl_oracle_segment_diagnostics(
        ctypes.c_int64(N), ctypes.c_int32(K), _ptr(seg), _ptr(ratio), _ptr(logp), _ptr(old_logp), _ptr(entropy),
        _ptr(mask), _ptr(adv), ctypes.c_double(eps_low), ctypes.c_double(eps_high), _ptr(out["count"]),
        _ptr(out["ratio_sum"]), _ptr(out["ratio_max"]), _ptr(out["clipped"]), _ptr(out["kl_sum"]),
        _ptr(out["ent_sum"]), _ptr(out["masked"]), ctypes.byref(oor))
    out["out_of_range"] = int(oor.value)
    return out


def pool_step(prev_len, new_len, hit_eos, seg_len, max_len):
    """One rollout step of Algorithm 1 (Sec. 3.1.1) -> dict with state, total_len, segments,
    unfinished_idx, experience_idx, exp_cu_seqlens, exp_truncated, counts (see the C source)."""
    prev = np.ascontiguousarray(prev_len, np.int32)
    new = np.ascontiguousarray(new_len, np.int32)
    eos = np.ascontiguousarray(hit_eos, np.uint8)
    B = prev.shape[0]
    state = np.zeros(B, np.uint8)
    total = np.zeros(B, np.int32)
    segs = np.zeros(B, np.int32)
    unf = np.zeros(max(B, 1), np.int32)
    exp = np.zeros(max(B, 1), np.int32)
    cu = np.zeros(B + 1, np.int64)
    trunc = np.zeros(max(B, 1), np.uint8)
    counts = np.zeros(5, np.int64)
    lib = _load()
    lib.ulorl_oracle_pool_step.restype = ctypes.c_int
    rc = lib.ulorl_oracle_pool_step(
        ctypes.c_int32(B), _ptr(prev), _ptr(new), _ptr(eos), ctypes.c_int32(seg_len), ctypes.c_int32(max_len),
        _ptr(state), _ptr(total), _ptr(segs), _ptr(unf), _ptr(exp), _ptr(cu), _ptr(trunc), _ptr(counts))
    if rc != 0:
        raise ValueError("oracle pool_step: bad seg_len / max_len / B")
    nu, ne = int(counts[0]), int(counts[1])
    return {"state": state, "total_len": total, "segments": segs, "unfinished_idx": unf[:nu],
            "experience_idx": exp[:ne], "exp_cu_seqlens": cu[:ne + 1], "exp_truncated": trunc[:ne],
            "counts": counts}
