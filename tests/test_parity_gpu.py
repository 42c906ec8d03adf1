"""GPU parity: the HIP decode step, called through the C ABI, against the fp64 CPU oracle.

Error measure (the whole `out` tensor of a case): max|y - ref| / max|ref|.
Bars: 1e-5 for fp32 storage, 2e-3 for fp16/bf16 storage with fp32 accumulation.  The worst per-row
ratio and the relative L2 error are recorded next to the gated figure (parity_errors.txt in the run-output folder).
"""
import numpy as np
import pytest

from paper_2105_04779_amd import workloads as wl
from helpers import TOL, err_report, fmt_report, gpu_out, make_layer, oracle_out, record, rel_err, to_device

pytestmark = pytest.mark.gpu


def run_case(w, *, lens=None, poison=True, flags=0, splits=0, row_groups=0, scale_q=None, elements=None, tol=None):
    W = wl.weights(w)
    H, Q, L = wl.batch(w, elements=elements, poison=False)
    if lens is not None:
        L = np.asarray(lens, dtype=np.int32)
    if scale_q is not None:
        Q = wl.round_to_storage(Q * np.float32(scale_q), w.dtype)
    Hp = H.copy()
    if poison:
        for b in range(H.shape[0]):
            Hp[b, L[b]:, :] = np.nan
    ref = oracle_out(w, W, H, Q, L)
    layer = make_layer(w, W, max_batch=H.shape[0], flags=flags)
    if splits:
        layer.set_splits(splits)
    if row_groups:
        layer.set_row_groups(row_groups)
    y = gpu_out(layer, w, Hp, Q, L)
    rep = err_report(y, ref)
    err = rep["tensor"]
    bar = tol or TOL[w.dtype]
    record(f"{w.name}: B={H.shape[0]} mfma={layer.uses_mfma} splits={splits} row_groups={row_groups} {fmt_report(rep)} bar={bar:g}")
    assert err <= bar, f"{w.name}: err {err:.3e} > {bar:g}"
    layer.close()
    return y


# ---- the tiny fp32 configuration ------------------------------------------------------------------
def test_c1_tiny_fp32():
    run_case(wl.WORKLOADS["c1_tiny_f32"])


def test_c1_tiny_fp32_ragged():
    run_case(wl.WORKLOADS["c1_tiny_f32"], lens=[32, 19])


# ---- small cases in every dtype: several tiles, ragged tails, odd shapes ---------------------------------
SMALL = [
    # dtype, B, beam, heads, d_m, d_k, n, lens
    ("f32", 3, 2, 4, 64, 16, 100, [100, 37, 1]),
    ("f32", 2, 3, 2, 128, 64, 70, [70, 33]),
    ("f16", 3, 4, 8, 512, 64, 200, [200, 129, 31]),
    ("bf16", 3, 4, 16, 1024, 64, 150, [150, 97, 64]),
    ("bf16", 2, 1, 16, 1024, 64, 130, [130, 65]),       # greedy / per-beam history: 16 rows per H
    ("bf16", 2, 6, 16, 1024, 64, 90, [90, 45]),         # beam 6: 96 rows, not a power of two
    ("f16", 2, 3, 8, 512, 64, 77, [77, 5]),             # 24 rows: not a multiple of 16
    ("bf16", 1, 4, 12, 768, 64, 140, [140]),            # GPT-2-small / BART-base width: rows of 1.5 KB
    ("bf16", 5, 4, 12, 768, 64, 210, [210, 16, 1, 97, 33]),
    ("f16", 3, 1, 12, 768, 64, 300, [300, 17, 255]),    # per-beam histories at that width: 12 rows per H
    ("bf16", 40, 2, 12, 768, 64, 50, None),             # 80 query rows: 2.5 row tiles in the projections
    ("f16", 2, 2, 4, 256, 64, 64, [64, 64]),
    ("f16", 2, 2, 4, 512, 128, 90, [90, 41]),           # head size 128: MFMA core between fp32-FMA projections
]


@pytest.mark.parametrize("dtype,B,beam,heads,d_m,d_k,n,lens", SMALL)
def test_small_cases(dtype, B, beam, heads, d_m, d_k, n, lens):
    w = wl.custom(f"small_{dtype}_{heads}x{beam}_{d_m}_{n}", dtype=dtype, B=B, beam=beam, heads=heads,
                  d_m=d_m, d_k=d_k, n=n, index=50)
    run_case(w, lens=lens)


@pytest.mark.parametrize("dtype,B,beam,heads,d_m,d_k,n,lens", SMALL[2:6])
def test_small_cases_generic_kernels(dtype, B, beam, heads, d_m, d_k, n, lens):
    from paper_2105_04779_amd import el_attn
    w = wl.custom(f"generic_{dtype}_{heads}x{beam}_{d_m}_{n}", dtype=dtype, B=B, beam=beam, heads=heads,
                  d_m=d_m, d_k=d_k, n=n, index=51)
    run_case(w, lens=lens, flags=el_attn.EL_FLAG_FORCE_GENERIC)


# ---- many query rows (several row blocks of every projection kernel, last one ragged) ----------------------
@pytest.mark.parametrize("dtype,B,beam,heads,d_m,n", [("bf16", 130, 4, 16, 1024, 40), ("f16", 150, 4, 8, 512, 33),
                                                      ("bf16", 513, 1, 16, 1024, 20)])
def test_many_rows_not_a_multiple_of_the_tile(dtype, B, beam, heads, d_m, n):
    w = wl.custom(f"rows_{dtype}_{B}x{beam}", dtype=dtype, B=B, beam=beam, heads=heads, d_m=d_m, d_k=64, n=n,
                  len_lo=1, len_hi=n, index=59)
    run_case(w)


# ---- degenerate cases ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,B,beam,heads,d_m,n", [("bf16", 1030, 1, 16, 1024, 20), ("bf16", 1100, 2, 12, 768, 18)])
def test_batches_beyond_the_flattened_cut(dtype, B, beam, heads, d_m, n):
    """More than 1024 batch elements are not cut as one tile list: one workgroup per (element, row block)."""
    w = wl.custom(f"wide_batch_{dtype}_{B}_{d_m}", dtype=dtype, B=B, beam=beam, heads=heads, d_m=d_m, d_k=64, n=n, index=55)
    lens = 1 + (np.arange(B) * 7) % n
    lens[0], lens[-1] = n, 1
    run_case(w, lens=lens)


def test_single_position_and_single_row():
    w = wl.custom("n1", dtype="bf16", B=2, beam=1, heads=16, d_m=1024, d_k=64, n=1, index=52)
    run_case(w, lens=[1, 1])
    w = wl.custom("len1_in_n64", dtype="f16", B=2, beam=4, heads=8, d_m=512, d_k=64, n=64, index=53)
    run_case(w, lens=[1, 64])


def test_lengths_null_means_full_length():
    import torch
    w = wl.custom("nolens", dtype="bf16", B=2, beam=4, heads=16, d_m=1024, d_k=64, n=96, index=54)
    W = wl.weights(w)
    H, Q, L = wl.batch(w)
    ref = oracle_out(w, W, H, Q, None)
    layer = make_layer(w, W)
    out = layer.decode_step(to_device(H, w.dtype), None, to_device(Q, w.dtype))
    torch.cuda.synchronize()
    assert rel_err(out.float().cpu().numpy(), ref) <= TOL[w.dtype]


def test_peaked_softmax_large_scores():
    # queries scaled up: scores of magnitude ~30 make each head select almost one position;
    # exercises the running-max bookkeeping (a plain exp without it would overflow fp16/fp32)
    # and the precision of the expanded queries (a single 16-bit plane of them misses the bar here).
    w = wl.custom("peaked", dtype="bf16", B=2, beam=4, heads=16, d_m=1024, d_k=64, n=200, index=55)
    run_case(w, lens=[200, 111], scale_q=24.0)
    w = wl.custom("peaked16", dtype="f16", B=2, beam=4, heads=8, d_m=512, d_k=64, n=200, index=59)
    run_case(w, lens=[200, 111], scale_q=24.0)
    w = wl.custom("peaked32", dtype="f32", B=2, beam=2, heads=4, d_m=64, d_k=16, n=80, index=56)
    run_case(w, lens=[80, 41], scale_q=24.0, tol=1e-4)


@pytest.mark.parametrize("splits", [1, 2, 3, 8])
def test_split_count_does_not_change_the_result(splits):
    w = wl.custom("splits", dtype="bf16", B=2, beam=4, heads=16, d_m=1024, d_k=64, n=300, index=57)
    run_case(w, lens=[300, 70], splits=splits)


@pytest.mark.parametrize("dtype,heads,d_m,beam", [("bf16", 16, 1024, 4), ("bf16", 16, 1024, 6), ("f16", 8, 512, 7), ("bf16", 12, 768, 4)])
@pytest.mark.parametrize("row_groups,splits", [(1, 1), (1, 3), (2, 1), (2, 2), (2, 5), (1, 8), (2, 8), (0, 0)])
def test_rows_per_workgroup_and_split_count_do_not_change_the_result(dtype, heads, d_m, beam, row_groups, splits):
    # every cut the automatic plan can choose: 16 or 32 rows per workgroup (one to seven row blocks that
    # share each span of tiles) times the number of spans, on ragged lengths with a short last tile
    w = wl.custom(f"cut_{dtype}_{heads}x{beam}", dtype=dtype, B=3, beam=beam, heads=heads, d_m=d_m, d_k=64, n=330, index=58)
    run_case(w, lens=[330, 161, 19], splits=splits, row_groups=row_groups)


def test_strided_batch_and_guard_bands():
    """H with a batch stride larger than n*d_m; canaries around `out` must survive."""
    import torch
    w = wl.custom("guard", dtype="f16", B=3, beam=4, heads=8, d_m=512, d_k=64, n=100, index=58)
    W = wl.weights(w)
    H, Q, L = wl.batch(w)
    L = np.asarray([100, 51, 77], dtype=np.int32)
    ref = oracle_out(w, W, H, Q, L)
    layer = make_layer(w, W)
    pad_rows = 7
    Hbig = torch.full((w.B, w.n + pad_rows, w.d_m), float("nan"), dtype=torch.float16, device="cuda")
    Hbig[:, :w.n] = to_device(H, w.dtype)
    for b in range(w.B):
        Hbig[b, L[b]:] = float("nan")
    Hview = Hbig[:, :w.n]                      # batch stride (n+7)*d_m
    guard = 4096
    buf = torch.full((guard + w.B * w.beam * w.d_m + guard,), 12345.0, dtype=torch.float32, device="cuda")
    out = buf[guard:guard + w.B * w.beam * w.d_m].view(w.B, w.beam, w.d_m)
    layer.decode_step(Hview, torch.from_numpy(L).cuda(), to_device(Q, w.dtype), out=out)
    torch.cuda.synchronize()
    assert torch.all(buf[:guard] == 12345.0) and torch.all(buf[-guard:] == 12345.0)
    assert rel_err(out.cpu().numpy(), ref) <= TOL[w.dtype]


def test_repeatable_bitwise():
    import torch
    w = wl.custom("repeat", dtype="bf16", B=4, beam=4, heads=16, d_m=1024, d_k=64, n=256, index=59)
    W = wl.weights(w)
    H, Q, L = wl.batch(w)
    L = np.asarray([256, 100, 200, 33], dtype=np.int32)
    layer = make_layer(w, W)
    Hd, Qd, Ld = to_device(H, w.dtype), to_device(Q, w.dtype), torch.from_numpy(L).cuda()
    a = layer.decode_step(Hd, Ld, Qd).clone()
    b = layer.decode_step(Hd, Ld, Qd).clone()
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_out_in_storage_dtype():
    import torch
    w = wl.custom("out16", dtype="f16", B=2, beam=4, heads=8, d_m=512, d_k=64, n=64, index=60)
    W = wl.weights(w)
    H, Q, L = wl.batch(w)
    ref = oracle_out(w, W, H, Q, L)
    layer = make_layer(w, W, out_dtype="f16")
    out = layer.decode_step(to_device(H, w.dtype), torch.from_numpy(L).cuda(), to_device(Q, w.dtype))
    torch.cuda.synchronize()
    assert out.dtype == torch.float16
    assert rel_err(out.float().cpu().numpy(), ref) <= 3e-3


def test_expand_query_matches_eq5():
    """Diagnostic export of a1+a2: EL-Q_i = (q W_i^Q + b_i^Q)(W_i^K)^T / sqrt(d_k), row r = i*beam + j."""
    import torch
    w = wl.custom("elq", dtype="bf16", B=2, beam=3, heads=16, d_m=1024, d_k=64, n=16, index=61)
    W = wl.weights(w)
    _, Q, _ = wl.batch(w)
    layer = make_layer(w, W)
    elq = layer.expand_query(to_device(Q, w.dtype))
    torch.cuda.synchronize()
    elq = elq.cpu().numpy().astype(np.float64)
    Wq, Wk, bq = (W[k].astype(np.float64) for k in ("Wq", "Wk", "bq"))
    Qp = Q.astype(np.float64) @ Wq + bq                           # [B, beam, hd]
    ref = np.empty_like(elq)
    for i in range(w.heads):
        sl = slice(i * w.d_k, (i + 1) * w.d_k)
        e = Qp[:, :, sl] @ Wk[:, sl].T / np.sqrt(w.d_k)            # [B, beam, d_m]
        for j in range(w.beam):
            ref[:, i * w.beam + j] = e[:, j]
    assert rel_err(elq, ref) <= 1e-5


# ---- several layers, one H ------------------------------------------------------------------------------------
def test_layers_with_own_weights_share_one_H():
    """Section 3.3 / Figure 1: every decoder layer reads the same encoder output; contexts do not interfere."""
    from dataclasses import replace
    import torch
    w = wl.custom("layers", dtype="bf16", B=3, beam=4, heads=16, d_m=1024, d_k=64, n=180, len_lo=40, len_hi=180, index=62)
    H, Q, L = wl.batch(w, poison=True)
    Hd, Qd = to_device(H, w.dtype), to_device(Q, w.dtype)
    Ld = torch.from_numpy(L).cuda()
    Ws = [wl.weights(w if k == 0 else replace(w, index=w.index + 1000 * k)) for k in range(3)]
    layers = [make_layer(w, W) for W in Ws]
    outs = [ly.decode_step(Hd, Ld, Qd) for ly in layers]          # all queued on one stream before any is checked
    torch.cuda.synchronize()
    for k, (W, y) in enumerate(zip(Ws, outs)):
        err = rel_err(y.float().cpu().numpy(), oracle_out(w, W, H, Q, L))
        record(f"layers: layer {k} err={err:.3e}")
        assert err <= TOL[w.dtype]
    assert rel_err(outs[1].float().cpu().numpy(), outs[0].float().cpu().numpy()) > 0.1   # different weights, different results


# ---- argument validation with a live context ---------------------------------------------------------------
def test_decode_step_argument_errors():
    import ctypes
    import torch
    from paper_2105_04779_amd import el_attn as ea
    w = wl.WORKLOADS["c1_tiny_f32"]
    W = wl.weights(w)
    layer = make_layer(w, W)
    H, Q, L = wl.batch(w)
    Hd, Qd = to_device(H, w.dtype), to_device(Q, w.dtype)
    out = torch.empty((w.B, w.beam, w.d_m), device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    I = ea.EL_ERR_INVALID_ARG
    ok_stride = w.n * w.d_m
    assert ea.el_attn_decode_step(layer.ctx, None, ok_stride, None, p(Qd), p(out), w.B, w.beam, w.n) == I
    assert ea.el_attn_decode_step(layer.ctx, p(Hd), ok_stride, None, None, p(out), w.B, w.beam, w.n) == I
    assert ea.el_attn_decode_step(layer.ctx, p(Hd), ok_stride, None, p(Qd), None, w.B, w.beam, w.n) == I
    assert ea.el_attn_decode_step(layer.ctx, p(Hd), ok_stride, None, p(Qd), p(out), w.B + 1, w.beam, w.n) == I
    assert ea.el_attn_decode_step(layer.ctx, p(Hd), ok_stride, None, p(Qd), p(out), w.B, w.beam + 1, w.n) == I
    assert ea.el_attn_decode_step(layer.ctx, p(Hd), ok_stride, None, p(Qd), p(out), w.B, w.beam, w.n + 1) == I
    assert ea.el_attn_decode_step(layer.ctx, p(Hd), ok_stride, None, p(Qd), p(out), 0, w.beam, w.n) == I
    assert ea.el_attn_decode_step(layer.ctx, p(Hd), ok_stride - 1, None, p(Qd), p(out), w.B, w.beam, w.n) == I
    assert ea.el_attn_set_splits(layer.ctx, ea.el_attn_max_splits() + 1) == I
    # workspace: too small / misaligned / missing
    need = ea.el_attn_workspace_bytes(layer.ctx)
    assert need > 0
    small = torch.empty(need, dtype=torch.uint8, device="cuda")
    assert ea.el_attn_bind_workspace(layer.ctx, p(small), need - 1) == ea.EL_ERR_WORKSPACE
    assert ea.el_attn_bind_workspace(layer.ctx, ctypes.c_void_p(small.data_ptr() + 8), need) == I
    st, ctx2 = ea.el_attn_prepare(layer.cfg, *[p(to_device(W[k], w.dtype)) for k in
                                               ("Wq", "bq", "Wk", "bk", "Wv", "bv", "Wo", "bo")])
    assert st == ea.EL_OK
    assert ea.el_attn_decode_step(ctx2, p(Hd), ok_stride, None, p(Qd), p(out), w.B, w.beam, w.n) == ea.EL_ERR_WORKSPACE
    assert ea.el_attn_destroy(ctx2) == ea.EL_OK
    # and the good call still works afterwards
    assert ea.el_attn_decode_step(layer.ctx, p(Hd), ok_stride, None, p(Qd), p(out), w.B, w.beam, w.n) == ea.EL_OK
    torch.cuda.synchronize()


# ---- the benchmark configurations at full size ---------------------------------------------------------------
FULL = ["c2_transformer_base_f16", "c3_bart_large_bf16", "c4_bart_large_b320_bf16",
        "c5_gpt2_medium_n512_bf16", "c5_gpt2_medium_n768_bf16", "c5_gpt2_medium_n1024_bf16"]
# the same two decoding set-ups at the width of the base-size models (12 heads, d_m 768: tile rows of 1.5 KB)
WIDTH_768 = {
    "w768_beam_search_bf16": wl.custom("w768_beam_search_bf16", dtype="bf16", B=64, beam=4, heads=12, d_m=768, d_k=64,
                                       n=1024, len_lo=512, len_hi=1024, index=70),
    "w768_per_beam_history_bf16": wl.custom("w768_per_beam_history_bf16", dtype="bf16", B=512, beam=1, heads=12,
                                            d_m=768, d_k=64, n=1024, index=71),
}
EVERY_ELEMENT = {"c2_transformer_base_f16", "c3_bart_large_bf16", "w768_beam_search_bf16"}   # the oracle does these whole batches in seconds


@pytest.mark.parametrize("name", FULL + sorted(WIDTH_768))
def test_full_size(name):
    """Run the whole batch on the GPU in the launch configuration the benchmark times (same B, n,
    lengths).  The two configurations with 64 sentences are compared in full; of the larger ones the
    oracle computes 16 batch elements (first, last, shortest, longest and twelve spread over the batch),
    element by element; the filler elements are finite noise of the same distribution."""
    import torch
    w = WIDTH_768[name] if name in WIDTH_768 else wl.WORKLOADS[name]
    W = wl.weights(w)
    L = wl.lengths(w)
    layer = make_layer(w, W)
    g = torch.Generator(device="cuda").manual_seed(1)
    td = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}[w.dtype]
    if name in EVERY_ELEMENT:
        sample = list(range(w.B))
    else:
        sample = sorted({0, w.B - 1, int(np.argmin(L)), int(np.argmax(L))} | {(k * w.B) // 13 for k in range(1, 13)})
    Hd = torch.randn((w.B, w.n, w.d_m), generator=g, device="cuda", dtype=torch.float32).to(td)
    Qd = torch.randn((w.B, w.beam, w.d_m), generator=g, device="cuda", dtype=torch.float32).to(td)
    Hs, Qs, Ls = wl.batch(w, elements=sample, poison=False)
    for k, b in enumerate(sample):
        Hk = Hs[k].copy()
        Hk[Ls[k]:] = np.nan
        Hd[b] = to_device(Hk, w.dtype)
        Qd[b] = to_device(Qs[k], w.dtype)
    out = layer.decode_step(Hd, torch.from_numpy(L).cuda(), Qd)
    torch.cuda.synchronize()
    y = out[sample].float().cpu().numpy()
    ref = oracle_out(w, W, Hs, Qs, Ls)
    rep = err_report(y, ref)
    record(f"{name}: {len(sample)} of {w.B} elements mfma={layer.uses_mfma} {fmt_report(rep)} bar={TOL[w.dtype]:g}")
    assert rep["tensor"] <= TOL[w.dtype]
    assert torch.isfinite(out).all()


# ---- hidden states with large-magnitude channels ------------------------------------------------------------------
def _outlier_case(compensate: bool, scales):
    """bf16 hidden states in which a few channels are far larger than the rest, as the outputs of trained
    encoders have.  With `compensate` the rows of W^K and W^V that read those channels are scaled down by the
    same factors (a trained model's keys and values stay of order one): the softmax keeps its usual spread
    and the case tests the range and precision of the products.  Without it the scores grow with the
    channels and the softmax sharpens."""
    w = wl.custom("outliers_" + ("comp" if compensate else "raw"), dtype="bf16", B=3, beam=4, heads=16, d_m=1024, d_k=64, n=260, index=61)
    W = dict(wl.weights(w))
    H, Q, L = wl.batch(w, poison=False)
    L = np.asarray([260, 133, 17], dtype=np.int32)
    cols = [5, 300, 777, 1023][:len(scales)]
    for c, sc in zip(cols, scales):
        H[:, :, c] = wl.round_to_storage(H[:, :, c] * np.float32(sc), w.dtype)
        if compensate:
            for k in ("Wk", "Wv"):
                Wk = W[k].copy()
                Wk[c, :] = wl.round_to_storage(Wk[c, :] / np.float32(sc), w.dtype)
                W[k] = Wk
    assert float(np.abs(H).max()) <= 65504.0
    ref = oracle_out(w, W, H, Q, L)
    Hp = H.copy()
    for b in range(w.B):
        Hp[b, L[b]:] = np.nan
    layer = make_layer(w, W)
    y = gpu_out(layer, w, Hp, Q, L)
    rep = err_report(y, ref)
    record(f"{w.name}: scales={list(scales)} max|H|={np.abs(H).max():.3g} mfma={layer.uses_mfma} {fmt_report(rep)} bar={TOL[w.dtype]:g}")
    assert rep["tensor"] <= TOL[w.dtype]
    # the input check finds nothing to report on this tensor
    import torch
    from paper_2105_04779_amd import el_attn
    got = el_attn.check_inputs(to_device(Hp, w.dtype), torch.from_numpy(L).cuda()).cpu().tolist()
    assert got[:3] == [0, 0, 0]
    layer.close()


def test_outlier_channels_with_matching_weights():
    _outlier_case(True, [1.0e2, 1.0e3, 3.0e3, 1.0e4])      # 1e4 x N(0,1): magnitudes up to ~4.5e4


def test_outlier_channels_with_plain_weights():
    _outlier_case(False, [1.0e2, 60.0])


def test_values_beyond_the_fp16_range_are_reported():
    """The 16-bit MFMA path rounds partial results and projections to fp16, so it documents |H| <= 65504.
    bf16 storage can hold more: the input check must flag exactly those values, on the tensor the step is
    then given, and the fp32 path (generic kernels, forced) must still compute that tensor."""
    import torch
    from paper_2105_04779_amd import el_attn
    w = wl.custom("beyond_f16", dtype="bf16", B=2, beam=2, heads=16, d_m=1024, d_k=64, n=70, index=62)
    W = wl.weights(w)
    H, Q, L = wl.batch(w, poison=False)
    L = np.asarray([70, 33], dtype=np.int32)
    H[0, 3, 17] = wl.round_to_storage(np.asarray([1.0e5], dtype=np.float32), w.dtype)[0]
    H[1, 20, 900] = wl.round_to_storage(np.asarray([-7.0e4], dtype=np.float32), w.dtype)[0]
    H[1, 50, 2] = wl.round_to_storage(np.asarray([9.0e4], dtype=np.float32), w.dtype)[0]          # beyond the length: not counted
    Hd = to_device(H, w.dtype)
    got = el_attn.check_inputs(Hd, torch.from_numpy(L).cuda()).cpu().tolist()
    assert got[0] == 0 and got[1] == 0 and got[2] == 2
    ref = oracle_out(w, W, H, Q, L)
    layer = make_layer(w, W, flags=el_attn.EL_FLAG_FORCE_GENERIC)
    y = gpu_out(layer, w, H, Q, L)
    rep = err_report(y, ref)
    record(f"{w.name}: generic path on |H| up to 1e5 {fmt_report(rep)}")
    assert rep["tensor"] <= TOL[w.dtype]
    layer.close()
