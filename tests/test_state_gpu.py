"""GPU parity of the state gather between decode steps (el_attn_gather_batch) against the oracle's
row-by-row definition: bit-exact, every dtype, ragged lengths, duplicates, strides, guard rows."""
import numpy as np
import pytest

from paper_2105_04779_amd import workloads as wl
from helpers import to_device, record

pytestmark = pytest.mark.gpu

SENTINEL = {"f32": 123.25, "f16": 123.25, "bf16": 123.0}


def bits(t):
    """device tensor -> numpy array of its raw bits (so NaN payloads compare too)"""
    import torch
    if t.dtype == torch.float32:
        return t.cpu().numpy().view(np.uint32)
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def run_gather(dtype, B_src, n, d_m, lens, index, *, B_dst=None, stride_pad=0, seed=0, lengths_none=False):
    import torch
    import oracle
    from paper_2105_04779_amd import el_attn
    rng = np.random.default_rng(1000 + seed)
    H = wl.round_to_storage(rng.standard_normal((B_src, n, d_m), dtype=np.float32), dtype)
    lens = None if lengths_none else np.asarray(lens, dtype=np.int32)
    index = np.asarray(index, dtype=np.int32)
    B_dst = len(index) if B_dst is None else B_dst
    before = np.full((B_dst, n, d_m), SENTINEL[dtype], dtype=np.float32)
    ref, ref_lens = oracle.gather_batch_reference(H, lens, index, before)

    def dev(x, pad):
        t = to_device(x, dtype)
        if not pad:
            return t
        big = torch.full((x.shape[0], n * d_m + pad), SENTINEL[dtype], dtype=t.dtype, device="cuda")
        big[:, :n * d_m] = t.reshape(x.shape[0], -1)
        return big[:, :n * d_m].unflatten(1, (n, d_m)), big

    src = dev(H, stride_pad)
    dst = dev(before, stride_pad)
    Hs, Hd = (src[0], dst[0]) if stride_pad else (src, dst)
    Ld = None if lens is None else torch.from_numpy(lens).cuda()
    Idx = torch.from_numpy(index).cuda()
    out_lens = torch.full((B_dst,), -5, dtype=torch.int32, device="cuda")
    el_attn.gather_batch(Hs, Ld, Idx, H_dst=Hd, lengths_dst=out_lens)
    torch.cuda.synchronize()
    assert np.array_equal(bits(Hd.contiguous()), bits(to_device(ref, dtype))), "gathered rows differ"
    assert np.array_equal(out_lens.cpu().numpy(), ref_lens)
    if stride_pad:   # the gap between batch elements is nobody's to write
        assert bool((dst[1][:, n * d_m:] == SENTINEL[dtype]).all())
    return ref_lens


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_compaction_and_reorder_small(dtype):
    d_m = 64 if dtype == "f32" else 512
    # drop finished sentences: survivors in order
    run_gather(dtype, 6, 70, d_m, [70, 1, 33, 64, 17, 70], [0, 2, 3, 5], seed=1)
    # beam re-order: parents repeat, some beams die out
    run_gather(dtype, 8, 45, d_m, [45, 40, 39, 45, 1, 2, 31, 32], [1, 1, 0, 3, 7, 7, 7, 6], seed=2)


def test_lengths_null_copies_everything():
    run_gather("bf16", 3, 33, 1024, None, [2, 0], lengths_none=True, seed=3)


def test_batch_strides_and_guard_bands():
    run_gather("f16", 4, 37, 512, [37, 5, 20, 36], [3, 3, 1], stride_pad=64, seed=4)


def test_index_outside_the_source_leaves_destination_untouched():
    lens = run_gather("bf16", 3, 20, 1024, [20, 7, 9], [5, 1, -2, 0], seed=5)
    assert lens.tolist() == [0, 7, 0, 20]


def test_row_count_not_a_multiple_of_the_block_and_single_row():
    run_gather("bf16", 2, 97, 1024, [97, 96], [1, 0], seed=6)
    run_gather("f32", 2, 1, 4, [1, 1], [1, 1, 0], seed=7)


def test_per_beam_histories_full_size_sampled():
    """GPT-2-medium-shaped per-beam histories (512 x 1024 x 1024 bf16, 1 GiB): sampled elements, bit-exact."""
    import torch
    from paper_2105_04779_amd import el_attn
    B, n, d_m = 512, 1024, 1024
    g = torch.Generator(device="cuda").manual_seed(77)
    H = torch.randn((B, n, d_m), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    rng = np.random.default_rng(78)
    lens = rng.integers(512, n, size=B, endpoint=True).astype(np.int32)
    index = rng.integers(0, B, size=B).astype(np.int32)           # every beam picks a parent
    dst = torch.full((B, n, d_m), 3.0, dtype=torch.bfloat16, device="cuda")
    Ld, Idx = torch.from_numpy(lens).cuda(), torch.from_numpy(index).cuda()
    out_lens = torch.empty((B,), dtype=torch.int32, device="cuda")
    el_attn.gather_batch(H, Ld, Idx, H_dst=dst, lengths_dst=out_lens)
    torch.cuda.synchronize()
    assert np.array_equal(out_lens.cpu().numpy(), lens[index])
    for i in list(rng.choice(B, size=12, replace=False)) + [0, B - 1]:
        L = int(lens[index[i]])
        assert torch.equal(dst[i, :L].view(torch.int16), H[int(index[i]), :L].view(torch.int16)), i
        assert bool((dst[i, L:] == 3.0).all()), i
    record(f"gather full size: B={B} n={n} d_m={d_m} sum_len={int(lens[index].sum())} bit-exact on 14 sampled elements")


# ---- input check: counts are integers, so the comparison with the oracle is exact ---------------------------------
@pytest.mark.parametrize("dtype,d_m", [("f32", 64), ("f16", 512), ("bf16", 1024)])
def test_check_inputs_counts_match_the_oracle(dtype, d_m):
    import torch
    import oracle
    from paper_2105_04779_amd import el_attn
    g = np.random.default_rng(31)
    B, n = 5, 77
    H = wl.round_to_storage(g.standard_normal((B, n, d_m), dtype=np.float32), dtype)
    lens = np.array([77, 33, 1, 0, 90], dtype=np.int32)          # two of them outside [1, n]
    # plant special values everywhere, valid rows and padding alike
    for _ in range(60):
        b, t, c = int(g.integers(B)), int(g.integers(n)), int(g.integers(d_m))
        H[b, t, c] = [np.nan, np.inf, -np.inf, 70000.0, -1.0e6, 65504.0, 65536.0][int(g.integers(7))]
    if dtype == "f16":
        H = np.where(np.abs(H) > 65504.0, np.sign(H) * np.inf, H).astype(np.float32)   # what fp16 storage would hold
    H = wl.round_to_storage(H, dtype) if dtype != "f16" else H
    ref = oracle.check_inputs_reference(H, lens)
    got = el_attn.check_inputs(to_device(H, dtype), torch.from_numpy(lens).cuda())
    torch.cuda.synchronize()
    assert got.cpu().tolist() == ref
    assert ref[0] == 2 and ref[1] > 0 and (dtype == "f16" or ref[2] > 0)
    # NULL lengths: every row of every element
    ref_all = oracle.check_inputs_reference(H, None)
    got_all = el_attn.check_inputs(to_device(H, dtype), None)
    torch.cuda.synchronize()
    assert got_all.cpu().tolist() == ref_all and ref_all[3] == B * n * d_m
    # a second call into the same report starts from zero again
    rep = el_attn.check_inputs(to_device(H, dtype), torch.from_numpy(lens).cuda(), report=got_all)
    torch.cuda.synchronize()
    assert rep.cpu().tolist() == ref


def test_check_inputs_on_a_clean_full_size_batch():
    import torch
    from paper_2105_04779_amd import el_attn
    w = wl.WORKLOADS["c3_bart_large_bf16"]
    L = wl.lengths(w)
    H = torch.randn((w.B, w.n, w.d_m), device="cuda", dtype=torch.float32).to(torch.bfloat16)
    H[:, -1, :] = float("nan")                                   # padding of every element shorter than n
    full = int((L == w.n).sum())
    got = el_attn.check_inputs(H, torch.from_numpy(L).cuda()).cpu().tolist()
    assert got == [0, full * w.d_m, 0, int(L.sum()) * w.d_m]
