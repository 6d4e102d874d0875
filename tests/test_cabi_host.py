"""Host-only checks of the C ABI: the library builds for gfx950, loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched (no GPU needed: every
call below fails validation, so no kernel is ever enqueued)."""
import ctypes
import os
import re

import pytest

import paper_2507_19766_amd as ulorl
from paper_2507_19766_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(ulorl_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = ulorl.load_library()
    names = declared_functions()
    assert "ulorl_token_loss_fwd" in names and "ulorl_token_loss_bwd" in names
    for n in names:
        assert hasattr(lib, n), n
    assert ulorl.version() >= 200
    assert not hasattr(lib, "ulorl_tune")            # no process-wide state: launch options travel per call
    assert ulorl.status_string(0) == "ok"
    assert "aligned" in ulorl.status_string(-4)


def test_workspace_query():
    assert ulorl.token_loss_workspace_bytes(0, 64, 1) == 0
    assert ulorl.token_loss_workspace_bytes(10, 64, 0) == 0
    assert ulorl.token_loss_workspace_bytes(10, 0, 1) == 0
    assert ulorl.token_loss_workspace_bytes(32768 * 65535 + 1, 64, 1) == 0
    a = ulorl.token_loss_workspace_bytes(131072, 4096, 1)
    b = ulorl.token_loss_workspace_bytes(131072, 4096, 1024)
    assert 0 < a < b < 5 << 20 and a % 256 == 0
    # the one-call path keeps 16 bytes per row and piece of the row: 10 pieces for 151936 fp32 logits
    c = ulorl.token_loss_workspace_bytes(131072, 151936, 1)
    assert c - a == 131072 * 16 * (10 - 1)
    # the sizes of the configurations the static-scratch entry point is documented with
    assert ulorl.token_loss_workspace_bytes(131072, 151936, 1) < 22 << 20


def _fwd(lib, logits=0x1000, dt=1, N=4, V=64, stride=64, y=0x2000, cu=0x3000, R=1, old=0x4000,
         adv=0x5000, params=None, loss=0x6000, logp=0x7000, ent=0x8000, lse=0x9000, g=0xa000,
         ws=0x10000, ws_bytes=1 << 20, use_params=True, launch=None, seg_stats=None):
    p = params or binding.Params()
    cp = p.to_c()
    vp = ctypes.c_void_p
    return lib.ulorl_token_loss_fwd(
        vp(logits), dt, N, V, stride, vp(y), vp(cu), R, None, vp(old), vp(adv),
        ctypes.byref(cp) if use_params else None, vp(loss), vp(logp), vp(ent), vp(lse), vp(g),
        None, None, None, None, None, None, seg_stats, vp(ws), ws_bytes, launch, None)


def test_forward_rejects_bad_arguments_on_the_host():
    lib = ulorl.load_library()
    P = binding.Params
    assert _fwd(lib, logits=0) == -1
    assert _fwd(lib, y=0) == -1
    assert _fwd(lib, lse=0) == -1
    assert _fwd(lib, loss=0) == -1
    assert _fwd(lib, cu=0) == -1
    assert _fwd(lib, old=0) == -1                                   # SAIS needs old_logp
    assert _fwd(lib, use_params=False) == -1
    assert _fwd(lib, N=0) == -2 and _fwd(lib, V=0) == -2 and _fwd(lib, stride=63) == -2
    assert _fwd(lib, R=0) == -2
    assert _fwd(lib, N=1 << 31) == -2
    assert _fwd(lib, N=32768 * 65535 + 1) == -2                      # more rows than the launch grids hold
    assert _fwd(lib, dt=2) == -3
    assert _fwd(lib, logits=0x1008) == -4
    assert _fwd(lib, V=60, stride=60) == -4                          # bf16 row of 120 bytes
    assert _fwd(lib, dt=0, V=62, stride=62) == -4                    # fp32 row of 248 bytes
    assert _fwd(lib, params=P(eps_low=-0.1)) == -5
    assert _fwd(lib, params=P(eps_high=float("nan"))) == -5
    assert _fwd(lib, params=P(tau=0.0)) == -5 and _fwd(lib, params=P(tau=1.5)) == -5
    assert _fwd(lib, params=P(sigma=float("nan"))) == -5
    assert _fwd(lib, params=P(is_mode=2)) == -5 and _fwd(lib, params=P(gate_mode=4)) == -5
    assert _fwd(lib, params=P(seg_len=-1)) == -5
    assert _fwd(lib, ws=0) == -6 and _fwd(lib, ws=0x10010) == -6 and _fwd(lib, ws_bytes=16) == -6


def test_launch_options_and_segment_stats_validate_on_the_host():
    lib = ulorl.load_library()
    L = binding._CLaunch
    four = ctypes.c_int32 * 4

    def launch(flags=0, spins=0, tile=0, group=0, reserved=(0, 0, 0, 0)):
        return ctypes.byref(L(flags, spins, tile, group, four(*reserved)))
    assert _fwd(lib, launch=launch(flags=4)) == -5            # unknown flag
    assert _fwd(lib, launch=launch(spins=-1)) == -5
    assert _fwd(lib, launch=launch(tile=2)) == -5 and _fwd(lib, launch=launch(group=65)) == -5
    assert _fwd(lib, launch=launch(reserved=(0, 0, 1, 0))) == -5
    assert _fwd(lib, launch=launch(flags=1, spins=5, tile=1, group=64), ws=0) == -6     # valid options: next check fails
    S = binding._CSegStats

    def seg(K=4, count=0x100, ws=0x20000, ws_bytes=1 << 20, reserved=0):
        return ctypes.byref(S(K, reserved, count, 0x200, 0x300, 0x400, 0x500, 0x600, 0x700, 0, ws, ws_bytes))
    assert _fwd(lib, seg_stats=seg(K=0)) == -2 and _fwd(lib, seg_stats=seg(K=1025)) == -2
    assert _fwd(lib, seg_stats=seg(reserved=1)) == -2
    assert _fwd(lib, seg_stats=seg(count=0)) == -1
    assert _fwd(lib, seg_stats=seg(ws=0)) == -6 and _fwd(lib, seg_stats=seg(ws=0x20010)) == -6
    assert _fwd(lib, seg_stats=seg(ws_bytes=64)) == -6
    assert _fwd(lib, seg_stats=seg(), ws=0) == -6             # valid: next check fails


def test_backward_rejects_bad_arguments_on_the_host():
    lib = ulorl.load_library()
    vp = ctypes.c_void_p

    def bwd(logits=0x1000, dt=1, N=4, V=64, stride=64, y=0x2000, lse=0x3000, g=0x4000, dz=0x5000):
        return lib.ulorl_token_loss_bwd(vp(logits), dt, N, V, stride, vp(y), vp(lse), vp(g), 1.0,
                                        vp(dz), None)
    assert bwd(logits=0) == -1 and bwd(y=0) == -1 and bwd(lse=0) == -1 and bwd(g=0) == -1
    assert bwd(dz=0) == -1
    assert bwd(N=-1) == -2 and bwd(stride=8) == -2 and bwd(N=32768 * 65535 + 1) == -2
    assert bwd(dt=7) == -3
    assert bwd(dz=0x5004) == -4 and bwd(logits=0x1002) == -4


def test_fused_entry_rejects_bad_arguments_on_the_host():
    lib = ulorl.load_library()
    vp = ctypes.c_void_p
    cp = binding.Params().to_c()

    def call(logits=0x1000, dz=0x20000, adv=0x5000, ws=0x10000, ws_bytes=1 << 20, N=4, stride=64, old=0x4000):
        return lib.ulorl_token_loss_fwd_bwd(
            vp(logits), 1, N, 64, stride, vp(0x2000), vp(0x3000), 1, None, vp(old), vp(adv), ctypes.byref(cp), 1.0,
            vp(0x6000), vp(0x7000), vp(0x8000), vp(0x9000), vp(0xa000), None, None, None, None, None, None, None,
            vp(dz), vp(ws), ws_bytes, None, None)
    assert call(logits=0) == -1 and call(dz=0) == -1 and call(adv=0) == -1 and call(old=0) == -1
    assert call(N=0) == -2 and call(stride=32) == -2
    assert call(dz=0x20008) == -4
    assert call(ws=0) == -6 and call(ws_bytes=64) == -6


def test_binding_refuses_cpu_tensors():
    import torch
    z = torch.zeros(2, 8)
    with pytest.raises(RuntimeError):
        ulorl.row_stats(z, torch.zeros(2, dtype=torch.int32))


def test_pool_step_rejects_bad_arguments_on_the_host():
    lib = ulorl.load_library()
    vp = ctypes.c_void_p

    def call(B=4, prev=0x1000, seg=16, mx=64, counts=0x9000):
        return lib.ulorl_segment_pool_step(B, vp(prev), vp(0x2000), vp(0x3000), seg, mx, vp(0x4000), vp(0x5000),
                                           vp(0x6000), vp(0x7000), vp(0x8000), vp(0xa000), vp(0xb000), vp(counts), None)
    assert call(prev=0) == -1 and call(counts=0) == -1
    assert call(B=0) == -2 and call(seg=0) == -2 and call(mx=0) == -2
    assert call(B=1 << 20, mx=1 << 20) == -2          # offsets of the packed batch would not fit in int32


def test_gemm_rejects_bad_arguments_on_the_host():
    lib = ulorl.load_library()
    vp = ctypes.c_void_p

    def call(a=0x1000, lda=64, ldb=64, M=16, N=16, K=64, ldc=16):
        return lib.ulorl_gemm_tn_bf16(vp(a), lda, vp(0x2000), ldb, M, N, K, vp(0x3000), ldc, None, None)
    assert call(a=0) == -1
    assert call(M=0) == -2 and call(K=60) == -2 and call(lda=32) == -2 and call(ldc=8) == -2
    assert call(lda=(1 << 22) + 8) == -2 and call(ldb=(1 << 22) + 8) == -2   # 32-bit tile offsets
    assert call(a=0x1008) == -4


def test_lmhead_workspace_query_rejects_bad_shapes():
    assert ulorl.lmhead_workspace_bytes(1024, 256, 4096, 2, 1024) > 0
    assert ulorl.lmhead_workspace_bytes(0, 256, 4096, 2, 1024) == 0
    assert ulorl.lmhead_workspace_bytes(1024, 256, 4096, 2, 1000) == 0     # chunk not a multiple of 64
