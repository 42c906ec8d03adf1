"""The decode step that allocates nothing (el_attn_decode_step_static: intermediates in a fixed array inside the
library's device code), through the C ABI, against el_attn_decode_step on the same inputs: two calls in a row,
the second with a smaller input, plus the size limit."""
import ctypes

import numpy as np
import pytest

from paper_2105_04779_amd import workloads as wl
from helpers import TOL, err_report, fmt_report, make_layer, oracle_out, record, to_device

pytestmark = pytest.mark.gpu


def _p(t):
    return ctypes.c_void_p(t.data_ptr())


def _both(ea, layer, w, H, Q, L):
    """out of decode_step (bound workspace) and of decode_step_static on the same device tensors."""
    import torch
    Hd, Qd = to_device(H, w.dtype), to_device(Q, w.dtype)
    Ld = torch.from_numpy(np.asarray(L, dtype=np.int32)).cuda()
    B, n = H.shape[0], H.shape[1]
    outs = []
    for fn in (ea.el_attn_decode_step, ea.el_attn_decode_step_static):
        out = torch.full((B, w.beam, w.d_m), float("nan"), device="cuda", dtype=torch.float32)
        st = fn(layer.ctx, _p(Hd), n * w.d_m, _p(Ld), _p(Qd), _p(out), B, w.beam, n, None)
        assert st == ea.EL_OK, ea.status_string(st)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
    return outs


@pytest.mark.parametrize("dtype,heads,d_m", [("bf16", 16, 1024), ("f32", 4, 64)])
def test_static_step_matches_the_step_with_a_bound_workspace(dtype, heads, d_m):
    from paper_2105_04779_amd import el_attn as ea
    d_k = d_m // heads
    w = wl.custom("noalloc_" + dtype, dtype=dtype, B=6, beam=4, heads=heads, d_m=d_m, d_k=d_k, n=150, index=63)
    W = wl.weights(w)
    layer = make_layer(w, W)
    # first call: the whole batch, ragged lengths with a short last tile
    H, Q, _ = wl.batch(w, poison=False)
    L = [150, 97, 64, 33, 1, 129]
    Hp = H.copy()
    for b in range(w.B):
        Hp[b, L[b]:] = np.nan
    y_ws, y_st = _both(ea, layer, w, Hp, Q, L)
    ref = oracle_out(w, W, H, Q, np.asarray(L, dtype=np.int32))
    rep_pair, rep_ref = err_report(y_st, y_ws), err_report(y_st, ref)
    record(f"{w.name} call 1: static vs bound {fmt_report(rep_pair)} | static vs oracle {fmt_report(rep_ref)}")
    assert rep_pair["tensor"] <= TOL[dtype] and rep_ref["tensor"] <= TOL[dtype]
    # second call, right after, on a smaller input (fewer batch elements, shorter keys): nothing of the
    # first call's intermediates may leak into it
    H2, Q2, L2 = Hp[1:3, :70].copy(), Q[1:3].copy(), [70, 41]
    for b in range(2):
        H2[b, L2[b]:] = np.nan
    y_ws2, y_st2 = _both(ea, layer, w, H2, Q2, L2)
    ref2 = oracle_out(w, W, np.nan_to_num(H2), Q2, np.asarray(L2, dtype=np.int32))
    rep_pair2, rep_ref2 = err_report(y_st2, y_ws2), err_report(y_st2, ref2)
    record(f"{w.name} call 2: static vs bound {fmt_report(rep_pair2)} | static vs oracle {fmt_report(rep_ref2)}")
    assert rep_pair2["tensor"] <= TOL[dtype] and rep_ref2["tensor"] <= TOL[dtype]
    layer.close()


def test_static_step_rejects_what_does_not_fit_and_checks_its_operands():
    import torch
    from paper_2105_04779_amd import el_attn as ea
    w = wl.custom("noalloc_big", dtype="bf16", B=64, beam=4, heads=16, d_m=1024, d_k=64, n=32, index=64)
    W = wl.weights(w)
    layer = make_layer(w, W)
    Hd = torch.zeros((w.B, w.n, w.d_m), device="cuda", dtype=torch.bfloat16)
    Qd = torch.zeros((w.B, w.beam, w.d_m), device="cuda", dtype=torch.bfloat16)
    out = torch.zeros((w.B, w.beam, w.d_m), device="cuda", dtype=torch.float32)
    call = lambda **k: ea.el_attn_decode_step_static(layer.ctx, k.get("H", _p(Hd)), w.n * w.d_m, None, _p(Qd), k.get("out", _p(out)),
                                                     k.get("B", w.B), w.beam, w.n, None)
    assert call() == ea.EL_ERR_WORKSPACE                       # 64 sentences x 4 beams need ~170 MB of intermediates
    assert call(B=8) == ea.EL_OK                               # 8 of them fit the 32 MiB array
    torch.cuda.synchronize()
    assert call(B=8, H=None) == ea.EL_ERR_INVALID_ARG
    assert call(B=8, out=ctypes.c_void_p(out.data_ptr() + 4)) == ea.EL_ERR_INVALID_ARG
    assert call(B=0) == ea.EL_ERR_INVALID_ARG
    layer.close()
