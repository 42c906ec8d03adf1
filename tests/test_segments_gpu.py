"""GPU parity of the segment form (section 3.2: EL-attention on the shared prefix and attention over each
beam's own continuation under one softmax), through the C ABI, against the fp64 CPU oracle.

Bars: the joined output and every segment's head outputs to the decode step's bar (max|y-ref|/max|ref|
<= 1e-5 fp32, 2e-3 for 16-bit storage); log(sum_t exp s_t), which is what a joint softmax consumes, to
1e-4 (fp32) / 5e-3 (16-bit: scores are formed from fp16 expanded queries) absolute, in natural-log units
of scores of order one.
"""
import numpy as np
import pytest

import oracle
from paper_2105_04779_amd import workloads as wl
from helpers import TOL, make_layer, record, rel_err, to_device

pytestmark = pytest.mark.gpu

LSE_TOL = {"f32": 1e-4, "f16": 5e-3, "bf16": 5e-3}


def _weights_with_visible_key_bias(w):
    W = wl.weights(w)
    W["bk"] = wl.round_to_storage(W["bk"] * np.float32(25.0), w.dtype)   # std 0.5: shifts scores by O(0.5)
    return W


def _inputs(w, seed, B, beam, n, lens):
    g = np.random.default_rng(seed)
    H = wl.round_to_storage(g.standard_normal((B, n, w.d_m), dtype=np.float32), w.dtype)
    Q = wl.round_to_storage(g.standard_normal((B, beam, w.d_m), dtype=np.float32), w.dtype)
    return H, Q, np.asarray(lens, dtype=np.int32)


def _seg_oracle(w, W, H, L, Q):
    return oracle.segment_reference(H, L, Q, W["Wq"], W["bq"], W["Wk"], W["bk"], W["Wv"], W["bv"],
                                    heads=w.heads, d_k=w.d_k)


def _seg_gpu(layer, w, H, L, Q, poison=True):
    import torch
    Hp = H.copy()
    if poison:
        for b in range(H.shape[0]):
            Hp[b, L[b]:, :] = np.nan
    A, S = layer.decode_segment(to_device(Hp, w.dtype), torch.from_numpy(L).cuda(), to_device(Q, w.dtype))
    torch.cuda.synchronize()
    return A, S


def _check_segment(tag, w, A, lse, refA, ref_lse):
    A, lse = A.cpu().numpy(), lse.cpu().numpy().astype(np.float64)
    eA = rel_err(A, refA)
    e_lse = float(np.abs(lse - ref_lse).max())
    record(f"{tag}: seg_A err={eA:.3e} lse err={e_lse:.3e}")
    assert eA <= TOL[w.dtype], f"{tag}: seg_A err {eA:.3e}"
    assert e_lse <= LSE_TOL[w.dtype], f"{tag}: log-sum-exp err {e_lse:.3e}"


CASES = [
    # dtype, heads, d_m, d_k, B, x, n1, n2, flags_generic, splits
    ("f32", 4, 64, 16, 2, 3, 70, 9, False, 0),
    ("bf16", 16, 1024, 64, 3, 4, 150, 20, False, 0),
    ("bf16", 16, 1024, 64, 2, 4, 200, 33, False, 3),      # prefix cut into key ranges
    ("f16", 8, 512, 64, 2, 5, 100, 17, False, 0),
    ("f16", 4, 512, 128, 2, 2, 90, 16, False, 0),         # MFMA core, fp32-FMA projections
    ("bf16", 16, 1024, 64, 2, 2, 80, 12, True, 0),        # generic kernels
    ("bf16", 12, 768, 64, 3, 4, 130, 21, False, 0),       # base-size width: tile rows of 1.5 KB
]


@pytest.mark.parametrize("dtype,heads,d_m,d_k,B,x,n1,n2,generic,splits", CASES)
def test_prefix_and_suffix_segments_joined(dtype, heads, d_m, d_k, B, x, n1, n2, generic, splits):
    import torch
    from paper_2105_04779_amd import el_attn
    w = wl.custom(f"seg_{dtype}_{heads}_{d_m}", dtype=dtype, B=B, beam=x, heads=heads, d_m=d_m, d_k=d_k, n=n1, index=70)
    W = _weights_with_visible_key_bias(w)
    g = np.random.default_rng(7)
    L1 = g.integers(max(1, n1 // 2), n1 + 1, B).astype(np.int32); L1[0] = n1
    L2 = g.integers(1, n2 + 1, B * x).astype(np.int32); L2[-1] = n2
    H1, Q, L1 = _inputs(w, 1, B, x, n1, L1)
    H2, _, L2 = _inputs(w, 2, B * x, 1, n2, L2)
    Q2 = Q.reshape(B * x, 1, d_m)
    layer = make_layer(w, W, max_batch=B * x, max_beam=x, max_n=max(n1, n2),
                       flags=el_attn.EL_FLAG_FORCE_GENERIC if generic else 0)
    if splits:
        layer.set_splits(splits)
    tag = f"segments {dtype} h{heads} d{d_m} dk{d_k} x{x} mfma={layer.uses_mfma} splits={splits}"

    seg1 = _seg_gpu(layer, w, H1, L1, Q)
    seg1 = (seg1[0].clone(), seg1[1].clone())
    seg2 = _seg_gpu(layer, w, H2, L2, Q2)
    ref1 = _seg_oracle(w, W, H1, L1, Q)
    ref2 = _seg_oracle(w, W, H2, L2, Q2)
    _check_segment(tag + " prefix", w, *seg1, *ref1)
    _check_segment(tag + " suffix", w, *seg2, *ref2)

    # joined on the device, against the definition on explicitly concatenated keys (one row per beam)
    out = layer.merge_segments([seg1, seg2], B, x)
    torch.cuda.synchronize()
    Hcat = np.zeros((B * x, n1 + n2, d_m), dtype=np.float32)
    Lcat = np.zeros(B * x, dtype=np.int32)
    for b in range(B):
        for j in range(x):
            r = b * x + j
            Hcat[r, :L1[b]] = H1[b, :L1[b]]
            Hcat[r, L1[b]:L1[b] + L2[r]] = H2[r, :L2[r]]
            Lcat[r] = L1[b] + L2[r]
    ref = oracle.mha_reference(Hcat, Lcat, Q2, W["Wq"], W["bq"], W["Wk"], W["bk"], W["Wv"], W["bv"],
                               W["Wo"], W["bo"], heads=heads, d_k=d_k).reshape(B, x, d_m)
    err = rel_err(out.float().cpu().numpy(), ref)
    record(f"{tag}: joined err={err:.3e}")
    assert err <= TOL[dtype]

    # one segment alone is the decode step
    alone = layer.merge_segments([seg1], B, x)
    step = layer.decode_step(to_device(H1, dtype), torch.from_numpy(L1).cuda(), to_device(Q, dtype))
    torch.cuda.synchronize()
    ref_step = oracle.mha_reference(H1, L1, Q, W["Wq"], W["bq"], W["Wk"], W["bk"], W["Wv"], W["bv"],
                                    W["Wo"], W["bo"], heads=heads, d_k=d_k)
    e_alone = rel_err(alone.float().cpu().numpy(), ref_step)
    e_step = rel_err(step.float().cpu().numpy(), ref_step)
    record(f"{tag}: one segment err={e_alone:.3e} (decode step {e_step:.3e})")
    assert e_alone <= TOL[dtype] and e_step <= TOL[dtype]
    layer.close()


def test_statistics_join_with_an_ordinary_attention_cache():
    # The per-beam continuation handled OUTSIDE the library (a caller's key/value cache): its log-sum-exp and head
    # outputs come from the definition (the oracle, as fp32 inputs); the prefix segment comes from the device.
    import torch
    w = wl.custom("seg_external", dtype="bf16", B=2, beam=4, heads=16, d_m=1024, d_k=64, n=120, index=71)
    W = _weights_with_visible_key_bias(w)
    B, x, n1, n2 = 2, 4, 120, 10
    H1, Q, L1 = _inputs(w, 3, B, x, n1, [120, 77])
    H2, _, L2 = _inputs(w, 4, B * x, 1, n2, [10, 3, 1, 7, 10, 2, 5, 9])
    Q2 = Q.reshape(B * x, 1, w.d_m)
    layer = make_layer(w, W, max_batch=B, max_beam=x, max_n=n1)
    seg1 = _seg_gpu(layer, w, H1, L1, Q)
    ext = _seg_oracle(w, W, H2, L2, Q2)
    seg2 = (torch.from_numpy(ext[0].astype(np.float32)).cuda(), torch.from_numpy(ext[1].astype(np.float32)).cuda())
    out = layer.merge_segments([seg1, seg2], B, x)
    torch.cuda.synchronize()
    ref1 = _seg_oracle(w, W, H1, L1, Q)
    ref = oracle.join_segments_reference([ref1, ext], W["Wo"], W["bo"], heads=w.heads, d_k=w.d_k).reshape(B, x, w.d_m)
    err = rel_err(out.float().cpu().numpy(), ref)
    record(f"segments joined with an external cache: err={err:.3e}")
    assert err <= TOL["bf16"]
    # the suffix really matters here: the prefix alone is a different answer
    alone = layer.merge_segments([seg1], B, x)
    torch.cuda.synchronize()
    assert rel_err(alone.float().cpu().numpy(), ref) > 10 * TOL["bf16"]
    layer.close()


def test_segment_arguments_are_validated():
    import torch
    from paper_2105_04779_amd import el_attn as ea
    w = wl.custom("seg_args", dtype="f16", B=2, beam=2, heads=8, d_m=512, d_k=64, n=40, index=72)
    W = wl.weights(w)
    layer = make_layer(w, W)
    A = torch.zeros((4, 512), dtype=torch.float32, device="cuda")
    S = torch.ones((4, 8), dtype=torch.float32, device="cuda")
    out = torch.zeros((2, 2, 512), dtype=torch.float32, device="cuda")
    p = lambda t: t.data_ptr()
    I = ea.EL_ERR_INVALID_ARG
    assert ea.el_attn_max_segments() == 4
    assert ea.el_attn_merge_segments(layer.ctx, 0, [p(A)], [p(S)], p(out), 2, 2) == I
    assert ea.el_attn_merge_segments(layer.ctx, 5, [p(A)] * 5, [p(S)] * 5, p(out), 2, 2) == I
    assert ea.el_attn_merge_segments(layer.ctx, 2, [p(A), None], [p(S), p(S)], p(out), 2, 2) == I
    assert ea.el_attn_merge_segments(layer.ctx, 1, [p(A)], [p(S)], None, 2, 2) == I
    assert ea.el_attn_merge_segments(layer.ctx, 1, [p(A)], [p(S)], p(out), 3, 2) == I       # beyond max_batch
    H = torch.zeros((2, 40, 512), dtype=torch.float16, device="cuda")
    Q = torch.zeros((2, 2, 512), dtype=torch.float16, device="cuda")
    assert ea.el_attn_decode_segment(layer.ctx, p(H), 40 * 512, None, p(Q), None, p(S), 2, 2, 40) == I
    assert ea.el_attn_decode_segment(layer.ctx, p(H), 40 * 512, None, p(Q), p(A), None, 2, 2, 40) == I
    assert ea.el_attn_decode_segment(layer.ctx, p(H), 40 * 512, None, p(Q), p(A), p(S), 2, 2, 41) == I
    # four equal segments joined are that segment
    sA, sS = layer.decode_segment(H + 1, None, Q + 1)
    one = layer.merge_segments([(sA, sS)], 2, 2)
    four = layer.merge_segments([(sA, sS)] * 4, 2, 2)
    torch.cuda.synchronize()
    assert torch.allclose(one, four, rtol=1e-5, atol=1e-6)
    layer.close()
