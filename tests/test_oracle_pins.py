"""Pins for the fp64 CPU oracle: everything here runs without a GPU.

The oracle (oracle/mha_oracle.c) is checked against things it did not produce:
a hand-worked example, closed forms, the paper's losslessness identity and its
two bias remarks (appendix B), torch's float64 multi-head attention on the CPU,
and invariances of the definition.
"""
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_problem(seed, B=2, beam=2, h=2, d_m=8, d_k=4, n=5, lengths=None, biases=True, scale=1.0):
    g = np.random.default_rng(seed)
    hd = h * d_k
    p = dict(
        H=g.standard_normal((B, n, d_m)),
        queries=g.standard_normal((B, beam, d_m)) * scale,
        Wq=g.standard_normal((d_m, hd)) / math.sqrt(d_m),
        Wk=g.standard_normal((d_m, hd)) / math.sqrt(d_m),
        Wv=g.standard_normal((d_m, hd)) / math.sqrt(d_m),
        Wo=g.standard_normal((hd, d_m)) / math.sqrt(hd),
        bq=g.standard_normal(hd) * 0.3 if biases else None,
        bk=g.standard_normal(hd) * 0.3 if biases else None,
        bv=g.standard_normal(hd) * 0.3 if biases else None,
        bo=g.standard_normal(d_m) * 0.3 if biases else None,
        lengths=None if lengths is None else np.asarray(lengths, dtype=np.int32),
    )
    return p, dict(heads=h, d_k=d_k)


def run(fn, p, kw, **override):
    q = dict(p)
    q.update(override)
    return fn(q["H"], q["lengths"], q["queries"], q["Wq"], q["bq"], q["Wk"], q["bk"],
              q["Wv"], q["bv"], q["Wo"], q["bo"], **kw)


# --------------------------------------------------------------------------------------
# hand-worked example (Eq. 1 reached from Eq. 2 with one head and identity projections)
# --------------------------------------------------------------------------------------
def _read_kv(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                out[k.strip()] = float(v)
    return out


def test_hand_worked_single_head_example():
    gold = _read_kv(os.path.join(GOLDEN, "single_head_two_positions.txt"))
    I = np.eye(2)
    H = np.array([[[1.0, 0.0], [0.0, 1.0]]])
    q = np.array([[[1.0, 0.0]]])
    for fn in (oracle.mha_reference, oracle.el_reference):
        out = fn(H, None, q, I, None, I, None, I, None, I, None, heads=1, d_k=2)
        assert out.shape == (1, 1, 2)
        assert abs(out[0, 0, 0] - gold["p0"]) < 1e-15
        assert abs(out[0, 0, 1] - gold["p1"]) < 1e-15


def test_scale_is_sqrt_dk_not_sqrt_dm():
    # Two heads of width 2 inside d_m = 4: identity projections make head i look at
    # coordinates (2i, 2i+1).  With Q = [a,0,b,0] and H rows e0, e2 the per-head
    # probabilities are logistic(a/sqrt(2)) and logistic(-b/sqrt(2)) (d_k = 2); a
    # sqrt(d_m) scale would give logistic(a/2) instead and fail.
    a, b = 1.3, -0.7
    I = np.eye(4)
    H = np.zeros((1, 2, 4)); H[0, 0, 0] = 1.0; H[0, 1, 2] = 1.0
    q = np.array([[[a, 0.0, b, 0.0]]])
    out = oracle.mha_reference(H, None, q, I, None, I, None, I, None, I, None, heads=2, d_k=2)
    p_head0_pos0 = 1.0 / (1.0 + math.exp(-a / math.sqrt(2)))   # head 0 sees K = [[1,0],[0,0]]
    p_head1_pos1 = 1.0 / (1.0 + math.exp(-b / math.sqrt(2)))   # head 1 sees K = [[0,0],[1,0]]
    # head 0 outputs p*V0 restricted to coords 0..1 -> [p_head0_pos0, 0]; head 1 -> [p_head1_pos1, 0]
    expect = np.array([p_head0_pos0, 0.0, p_head1_pos1, 0.0])
    assert np.allclose(out[0, 0], expect, atol=1e-15, rtol=0)


# --------------------------------------------------------------------------------------
# appendix B: losslessness identity and the two bias remarks
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,lengths", [(1, None), (2, [2, 1]), (5, [5, 3]), (7, [1, 7])])
@pytest.mark.parametrize("h,d_m,d_k", [(2, 8, 4), (3, 6, 2), (2, 8, 3)])
def test_losslessness_identity_eq6_equals_eq9(n, lengths, h, d_m, d_k):
    p, kw = rand_problem(11 + n, h=h, d_m=d_m, d_k=d_k, n=n, lengths=lengths)
    a = run(oracle.mha_reference, p, kw)
    b = run(oracle.el_reference, p, kw)
    assert np.max(np.abs(a - b)) <= 1e-12


def test_key_bias_cancels_in_softmax():
    p, kw = rand_problem(3, n=6, lengths=[6, 4])
    base = run(oracle.mha_reference, p, kw)
    g = np.random.default_rng(0)
    for bk in (None, np.zeros_like(p["bk"]), 100.0 * g.standard_normal(p["bk"].shape)):
        other = run(oracle.mha_reference, p, kw, bk=bk)
        assert np.max(np.abs(other - base)) <= 1e-11
        other = run(oracle.el_reference, p, kw, bk=bk)
        assert np.max(np.abs(other - base)) <= 1e-11


def test_value_bias_passes_through_as_bv_times_wo():
    p, kw = rand_problem(4, n=6, lengths=[6, 2])
    with_bv = run(oracle.mha_reference, p, kw)
    without = run(oracle.mha_reference, p, kw, bv=None)
    shift = p["bv"] @ p["Wo"]                     # sum_i b_i^V W_i^O, the same for every row
    assert np.max(np.abs((with_bv - without) - shift[None, None, :])) <= 1e-13


def test_output_bias_added_once_per_row():
    p, kw = rand_problem(5, n=4)
    a = run(oracle.mha_reference, p, kw)
    b = run(oracle.mha_reference, p, kw, bo=None)
    assert np.max(np.abs((a - b) - p["bo"][None, None, :])) <= 1e-14


# --------------------------------------------------------------------------------------
# closed forms
# --------------------------------------------------------------------------------------
def test_length_one_ignores_the_query():
    p, kw = rand_problem(6, n=4, lengths=[1, 1])
    out = run(oracle.mha_reference, p, kw)
    for b in range(2):
        expect = (p["H"][b, 0] @ p["Wv"] + p["bv"]) @ p["Wo"] + p["bo"]
        for j in range(2):
            assert np.max(np.abs(out[b, j] - expect)) <= 1e-13


def test_zero_query_projection_gives_uniform_attention():
    p, kw = rand_problem(7, n=6, lengths=[6, 4])
    out = run(oracle.mha_reference, p, kw, Wq=np.zeros_like(p["Wq"]), bq=None)
    for b, L in enumerate([6, 4]):
        expect = (p["H"][b, :L].mean(axis=0) @ p["Wv"] + p["bv"]) @ p["Wo"] + p["bo"]
        assert np.max(np.abs(out[b] - expect[None, :])) <= 1e-13


def test_huge_query_selects_argmax_position_per_head():
    p, kw = rand_problem(8, B=1, beam=1, h=2, d_m=8, d_k=4, n=6, scale=1e4)
    out = run(oracle.mha_reference, p, kw)
    h, d_k = 2, 4
    q = p["queries"][0, 0] @ p["Wq"] + p["bq"]
    K = p["H"][0] @ p["Wk"] + p["bk"]
    V = p["H"][0] @ p["Wv"] + p["bv"]
    a = np.zeros(h * d_k)
    for i in range(h):
        sl = slice(i * d_k, (i + 1) * d_k)
        t = int(np.argmax(K[:, sl] @ q[sl]))
        a[sl] = V[t, sl]
    expect = a @ p["Wo"] + p["bo"]
    assert np.max(np.abs(out[0, 0] - expect)) <= 1e-9


# --------------------------------------------------------------------------------------
# library cross-check: torch's own multi-head attention in float64 on the CPU
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("B,beam,h,d_k,n,lengths", [
    (2, 2, 4, 4, 9, [9, 5]),
    (3, 1, 2, 8, 17, [1, 17, 11]),
    (1, 3, 8, 8, 33, None),
])
def test_against_torch_float64_multi_head_attention(B, beam, h, d_k, n, lengths):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    d_m = h * d_k
    p, kw = rand_problem(20 + n, B=B, beam=beam, h=h, d_m=d_m, d_k=d_k, n=n, lengths=lengths)
    ours = run(oracle.mha_reference, p, kw)

    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    N = B * beam
    query = t(p["queries"].reshape(1, N, d_m))                          # [L=1, N, E]
    key = t(np.repeat(p["H"], beam, axis=0).transpose(1, 0, 2).copy())  # [S, N, E]
    in_w = t(np.concatenate([p["Wq"].T, p["Wk"].T, p["Wv"].T], axis=0))
    in_b = t(np.concatenate([p["bq"], p["bk"], p["bv"]]))
    mask = None
    if lengths is not None:
        L = np.repeat(np.asarray(lengths), beam)
        mask = t(np.arange(n)[None, :] >= L[:, None])
    ref, _ = F.multi_head_attention_forward(
        query, key, key, d_m, h, in_w, in_b, None, None, False, 0.0,
        t(p["Wo"].T.copy()), t(p["bo"]), training=False, key_padding_mask=mask, need_weights=False)
    ref = ref.numpy().reshape(B, beam, d_m)
    assert np.max(np.abs(ours - ref)) <= 1e-12


# --------------------------------------------------------------------------------------
# invariances of the definition
# --------------------------------------------------------------------------------------
def test_invariances():
    p, kw = rand_problem(9, B=3, beam=3, h=2, d_m=8, d_k=4, n=7, lengths=[7, 4, 2])
    base = run(oracle.mha_reference, p, kw)

    # batch elements are independent: solving one alone gives the same rows
    for b in range(3):
        solo = run(oracle.mha_reference, p, kw, H=p["H"][b:b + 1], queries=p["queries"][b:b + 1],
                   lengths=p["lengths"][b:b + 1])
        assert np.array_equal(solo[0], base[b])

    # permuting beams permutes outputs; identical queries give identical rows
    perm = [2, 0, 1]
    out = run(oracle.mha_reference, p, kw, queries=p["queries"][:, perm])
    assert np.array_equal(out, base[:, perm])
    same = np.repeat(p["queries"][:, :1], 3, axis=1)
    out = run(oracle.mha_reference, p, kw, queries=same)
    assert np.array_equal(out[:, 0], out[:, 1]) and np.array_equal(out[:, 0], out[:, 2])

    # permuting the valid positions of H[b] leaves the result unchanged (up to summation order)
    H2 = p["H"].copy()
    H2[0, :7] = H2[0, [3, 1, 6, 0, 5, 2, 4]]
    H2[1, :4] = H2[1, [2, 3, 0, 1]]
    out = run(oracle.mha_reference, p, kw, H=H2)
    assert np.max(np.abs(out - base)) <= 1e-13

    # storage beyond the valid prefix is never read
    H3 = p["H"].copy()
    H3[1, 4:] = np.nan
    H3[2, 2:] = np.inf
    for fn in (oracle.mha_reference, oracle.el_reference):
        out = run(fn, p, kw, H=H3)
        assert np.all(np.isfinite(out))
    assert np.array_equal(run(oracle.mha_reference, p, kw, H=H3), base)


def test_rejects_bad_lengths():
    p, kw = rand_problem(10, n=4)
    for bad in ([0, 4], [5, 1], [-1, 2]):
        with pytest.raises(ValueError):
            run(oracle.mha_reference, p, kw, lengths=np.asarray(bad, dtype=np.int32))


def test_thread_count_reported():
    assert oracle.num_threads() >= 1


# ---- state gather: the loop-by-definition oracle against numpy's own indexing on a case where both apply ----
def test_gather_reference_equals_fancy_indexing_on_full_lengths():
    import oracle
    rng = np.random.default_rng(5)
    H = rng.standard_normal((5, 7, 8)).astype(np.float32)
    idx = np.array([4, 0, 0, 3], dtype=np.int32)
    before = np.full((4, 7, 8), -7.0, dtype=np.float32)
    out, lens = oracle.gather_batch_reference(H, None, idx, before)
    assert np.array_equal(out, H[idx]) and np.array_equal(lens, np.full(4, 7, dtype=np.int32))
    # ragged: rows at or beyond the length keep the old contents, rows below it are the source's
    L = np.array([7, 1, 3, 0, 5], dtype=np.int32)
    out, lens = oracle.gather_batch_reference(H, L, idx, before)
    assert np.array_equal(lens, L[idx])
    for i, s in enumerate(idx):
        assert np.array_equal(out[i, :L[s]], H[s, :L[s]]) and np.all(out[i, L[s]:] == -7.0)
    # an index outside the source leaves its destination alone
    out, lens = oracle.gather_batch_reference(H, L, np.array([9, -1, 2], dtype=np.int32), before[:3])
    assert np.all(out[0] == -7.0) and np.all(out[1] == -7.0) and lens.tolist() == [0, 0, 3]


# --------------------------------------------------------------------------------------
# segment form (section 3.2: one softmax over a shared prefix and per-beam continuations)
# --------------------------------------------------------------------------------------
def _segment(p, kw, **override):
    q = dict(p)
    q.update(override)
    return oracle.segment_reference(q["H"], q["lengths"], q["queries"], q["Wq"], q["bq"], q["Wk"], q["bk"],
                                    q["Wv"], q["bv"], **kw)


def test_one_segment_joined_is_plain_attention():
    p, kw = rand_problem(41, B=2, beam=3, h=2, d_m=8, d_k=4, n=6, lengths=[6, 4])
    seg = _segment(p, kw)
    got = oracle.join_segments_reference([seg], p["Wo"], p["bo"], **kw)
    ref = run(oracle.mha_reference, p, kw).reshape(got.shape)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_segment_log_sum_exp_is_that_of_the_biased_scores():
    # scores retyped with einsum over explicitly built keys; scipy's logsumexp as the independent routine
    from scipy.special import logsumexp
    p, kw = rand_problem(42, B=2, beam=2, h=2, d_m=8, d_k=4, n=5)
    _, lse = _segment(p, kw)
    K = (p["H"] @ p["Wk"] + p["bk"]).reshape(2, 5, 2, 4)
    Q = (p["queries"] @ p["Wq"] + p["bq"]).reshape(2, 2, 2, 4)
    s = np.einsum("bjic,btic->bjit", Q, K) / 2.0   # sqrt(d_k) = 2
    np.testing.assert_allclose(lse, logsumexp(s, axis=-1).reshape(4, 2), rtol=1e-13)
    # the key bias shifts it by Q_i . b_i^K / sqrt(d_k) (Eq. 7) and leaves seg_A alone
    A0, l0 = _segment(p, kw, bk=None)
    A1, l1 = _segment(p, kw)
    shift = np.einsum("bjic,ic->bji", Q, p["bk"].reshape(2, 4)).reshape(4, 2) / 2.0
    np.testing.assert_allclose(l1 - l0, shift, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(A1, A0, rtol=1e-12, atol=1e-14)


def test_single_key_segment_returns_its_value_row_and_its_score():
    p, kw = rand_problem(43, B=1, beam=2, h=2, d_m=8, d_k=4, n=3, lengths=[1])
    A, lse = _segment(p, kw)
    v = p["H"][0, 0] @ p["Wv"] + p["bv"]
    np.testing.assert_allclose(A, np.stack([v, v]), rtol=1e-13)
    k = (p["H"][0, 0] @ p["Wk"] + p["bk"]).reshape(2, 4)
    Q = (p["queries"][0] @ p["Wq"] + p["bq"]).reshape(2, 2, 4)
    np.testing.assert_allclose(lse, (Q * k).sum(-1) / 2.0, rtol=1e-13)


@pytest.mark.parametrize("x,n1,n2", [(1, 4, 3), (3, 5, 2), (2, 1, 1)])
def test_prefix_and_per_beam_suffix_joined_equal_attention_over_the_concatenation(x, n1, n2):
    # shared prefix scored as (B, beam=x); each beam's own continuation as (B*x, beam=1)
    B = 2
    p, kw = rand_problem(44 + x, B=B, beam=x, h=2, d_m=8, d_k=4, n=n1,
                         lengths=np.random.default_rng(x).integers(1, n1 + 1, B))
    g = np.random.default_rng(100 + x)
    H2 = g.standard_normal((B * x, n2, 8))
    len2 = g.integers(1, n2 + 1, B * x).astype(np.int32)
    seg1 = _segment(p, kw)
    seg2 = _segment(p, kw, H=H2, lengths=len2, queries=p["queries"].reshape(B * x, 1, 8))
    got = oracle.join_segments_reference([seg1, seg2], p["Wo"], p["bo"], **kw)
    # the definition on explicitly concatenated keys, one row per beam
    ncat = n1 + n2
    Hcat = np.zeros((B * x, ncat, 8))
    lcat = np.zeros(B * x, dtype=np.int32)
    for b in range(B):
        for j in range(x):
            r = b * x + j
            l1, l2 = int(p["lengths"][b]), int(len2[r])
            Hcat[r, :l1] = p["H"][b, :l1]
            Hcat[r, l1:l1 + l2] = H2[r, :l2]
            lcat[r] = l1 + l2
    ref = run(oracle.mha_reference, p, kw, H=Hcat, lengths=lcat, queries=p["queries"].reshape(B * x, 1, 8))
    np.testing.assert_allclose(got, ref.reshape(got.shape), rtol=1e-11, atol=1e-12)
    # dropping the key bias from ONE segment only must change the result (it no longer cancels)
    seg2_nobk = _segment(p, kw, H=H2, lengths=len2, queries=p["queries"].reshape(B * x, 1, 8), bk=None)
    bad = oracle.join_segments_reference([seg1, seg2_nobk], p["Wo"], p["bo"], **kw)
    assert np.abs(bad - got).max() > 1e-4


def test_check_inputs_reference_counts_exactly_what_was_planted():
    # expected counts are known by construction, not computed by the function under test
    g = np.random.default_rng(60)
    B, n, d = 3, 7, 8
    H = g.standard_normal((B, n, d)).astype(np.float32)
    lens = np.array([7, 4, 0], dtype=np.int32)            # one length outside [1, n]
    H[0, 2, 3] = np.nan; H[0, 6, 0] = np.inf; H[1, 3, 7] = -np.inf      # three non-finite, all in valid rows
    H[1, 0, 1] = 70000.0; H[0, 0, 0] = -65505.0                          # two beyond the fp16 range
    H[0, 1, 1] = 65504.0                                                 # exactly representable: not counted
    H[1, 5, 2] = np.nan; H[2, 0, 0] = 1e9                                # beyond the lengths: never looked at
    assert oracle.check_inputs_reference(H, lens) == [1, 3, 2, (7 + 4 + 0) * d]
    assert oracle.check_inputs_reference(H, None) == [0, 4, 3, 3 * 7 * d]
    assert oracle.check_inputs_reference(H, np.array([9, -2, 7])) == [2, 2, 2, (7 + 0 + 7) * d]   # element 1 skipped, element 2 walked
