"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ea():
    from paper_2105_04779_amd import el_attn
    return el_attn


def test_library_exports_every_declared_symbol(ea):
    header = open(os.path.join(ROOT, "include", "el_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(el_attn_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found in the header"
    assert declared == set(ea.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(ea.lib, name), f"{name} is declared but not exported"


def test_version_and_strings(ea):
    assert ea.el_attn_version() >= 100
    assert ea.el_attn_max_splits() >= 1
    assert ea.status_string(ea.EL_OK) == "ok"
    for s in range(1, 6):
        assert ea.status_string(s) not in ("ok", "unknown status")
    assert ea.status_string(99) == "unknown status"


def _cfg(ea, **kw):
    base = dict(heads=4, d_model=64, d_k=16, dtype=ea.EL_F32, out_dtype=ea.EL_F32,
                max_batch=2, max_beam=2, max_n=32, flags=0)
    base.update(kw)
    return ea.ElAttnConfig(*[base[k] for k in ("heads", "d_model", "d_k", "dtype", "out_dtype",
                                               "max_batch", "max_beam", "max_n", "flags")])


FAKE = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first


def test_prepare_rejects_bad_arguments_before_any_device_work(ea):
    I, U = ea.EL_ERR_INVALID_ARG, ea.EL_ERR_UNSUPPORTED
    ok = _cfg(ea)
    st, _ = ea.el_attn_prepare(ok, None, None, FAKE, None, FAKE, None, FAKE, None)
    assert st == I
    st, _ = ea.el_attn_prepare(ok, FAKE, None, FAKE, None, FAKE, None, None, None)
    assert st == I
    for bad in (dict(heads=0), dict(d_model=0), dict(d_k=-1), dict(max_batch=0), dict(max_beam=0), dict(max_n=0)):
        st, _ = ea.el_attn_prepare(_cfg(ea, **bad), FAKE, None, FAKE, None, FAKE, None, FAKE, None)
        assert st == I, bad
    for bad in (dict(d_k=8), dict(dtype=7), dict(out_dtype=9), dict(dtype=ea.EL_F16, out_dtype=ea.EL_BF16),
                dict(d_model=16384, heads=256, d_k=64)):
        st, _ = ea.el_attn_prepare(_cfg(ea, **bad), FAKE, None, FAKE, None, FAKE, None, FAKE, None)
        assert st == U, bad


def test_null_context_is_rejected_everywhere(ea):
    I = ea.EL_ERR_INVALID_ARG
    assert ea.el_attn_workspace_bytes(None) == 0
    assert ea.el_attn_bind_workspace(None, FAKE, 1024) == I
    assert ea.el_attn_decode_step(None, FAKE, 64, None, FAKE, FAKE, 1, 1, 1) == I
    assert ea.el_attn_expand_query(None, FAKE, FAKE, 1, 1) == I
    assert ea.el_attn_set_splits(None, 1) == I
    assert ea.el_attn_set_row_groups(None, 1) == I
    assert ea.el_attn_uses_mfma(None) == 0
    assert ea.el_attn_core_timing_enable(None, 4) == I
    assert ea.el_attn_core_timing_read(None, 4)[0] == I
    assert ea.el_attn_destroy(None) == I
    assert ea.el_attn_decode_segment(None, FAKE, 64, None, FAKE, FAKE, FAKE, 1, 1, 1) == I
    assert ea.el_attn_merge_segments(None, 1, [FAKE], [FAKE], FAKE, 1, 1) == I
    assert 1 <= ea.el_attn_max_segments() <= 16


def test_prepare_without_a_device_reports_hip_error(ea):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    st, ctx = ea.el_attn_prepare(_cfg(ea), FAKE, None, FAKE, None, FAKE, None, FAKE, None)
    assert st == ea.EL_ERR_HIP
    assert not ctx.value


def test_gather_batch_rejects_bad_arguments_before_any_device_work(ea):
    I = ea.EL_ERR_INVALID_ARG
    A, B, X = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x20000), ctypes.c_void_p(0x30000)   # never dereferenced

    def call(dtype=ea.EL_BF16, d_model=1024, src=A, sstride=64 * 1024, lsrc=None, bsrc=4,
             dst=B, dstride=64 * 1024, ldst=None, bdst=3, index=X, n=64):
        return ea.el_attn_gather_batch(dtype, d_model, src, sstride, lsrc, bsrc, dst, dstride, ldst, bdst, index, n)

    assert call(src=None) == I and call(dst=None) == I and call(index=None) == I
    assert call(dtype=5) == I
    for bad in (dict(d_model=0), dict(bsrc=0), dict(bdst=0), dict(n=0), dict(bdst=70000)):
        assert call(**bad) == I, bad
    assert call(sstride=64 * 1024 - 8) == I and call(dstride=100) == I          # shorter than n rows
    assert call(d_model=1020) == I                                              # 2040-byte rows: not a multiple of 16
    assert call(dtype=ea.EL_F32, d_model=6, sstride=6 * 64, dstride=6 * 64) == I
    assert call(src=ctypes.c_void_p(0x10008)) == I                              # misaligned
    assert call(sstride=64 * 1024 + 4) == I                                     # batch stride breaks the 16-byte alignment


def test_step_operands_are_validated_on_the_host(ea):
    """The checks decode_step applies to its operands, through the context-free entry point:
    shapes, strides and, on the MFMA path, 16-byte alignment.  Fake pointers, never dereferenced."""
    I, OK = ea.EL_ERR_INVALID_ARG, ea.EL_OK
    H, Q, O, L = (ctypes.c_void_p(v) for v in (0x100000, 0x200000, 0x300000, 0x400000))
    cfg = _cfg(ea, heads=16, d_model=1024, d_k=64, dtype=ea.EL_BF16, max_batch=8, max_beam=4, max_n=128)

    def call(mfma=1, H=H, stride=128 * 1024, lengths=L, queries=Q, out=O, B=8, beam=4, n=128, cfg=cfg):
        return ea.el_attn_check_step_operands(cfg, mfma, H, stride, lengths, queries, out, B, beam, n)

    assert call() == OK and call(lengths=None) == OK and call(mfma=0) == OK
    for bad in (dict(H=None), dict(queries=None), dict(out=None), dict(B=0), dict(B=9), dict(beam=5), dict(n=0), dict(n=129),
                dict(stride=128 * 1024 - 8)):
        assert call(**bad) == I, bad
    off = lambda p, k: ctypes.c_void_p(p.value + k)
    # MFMA path: 16-byte pieces
    for bad in (dict(H=off(H, 2)), dict(H=off(H, 8)), dict(queries=off(Q, 2)), dict(out=off(O, 4)), dict(out=off(O, 8)),
                dict(stride=128 * 1024 + 4), dict(stride=128 * 1024 + 1), dict(lengths=off(L, 2))):
        assert call(**bad) == I, bad
    assert call(stride=128 * 1024 + 8) == OK                     # 16 bytes more between batch elements
    # generic path: element alignment only
    assert call(mfma=0, H=off(H, 2), queries=off(Q, 2), stride=128 * 1024 + 1) == OK
    assert call(mfma=0, H=off(H, 1)) == I and call(mfma=0, out=off(O, 2)) == I and call(mfma=0, lengths=off(L, 1)) == I
    # a shape without MFMA kernels cannot be asked for their rules
    c640 = _cfg(ea, heads=10, d_model=640, d_k=64, dtype=ea.EL_BF16, max_batch=8, max_beam=4, max_n=128)
    assert call(cfg=c640, stride=128 * 640) == ea.EL_ERR_UNSUPPORTED
    assert call(cfg=c640, mfma=0, stride=128 * 640) == OK
    c768 = _cfg(ea, heads=12, d_model=768, d_k=64, dtype=ea.EL_BF16, max_batch=8, max_beam=4, max_n=128)
    assert call(cfg=c768, stride=128 * 768) == OK                # rows of 1.5 KB have MFMA kernels too
    assert ea.lib.el_attn_check_step_operands(None, 1, H, 1, L, Q, O, 1, 1, 1) == I


def test_plan_preview_on_the_benchmark_shapes(ea):
    """The automatic cut of the work, on a 256-unit device: host arithmetic only."""
    def plan(B, beam, heads, d_m, n):
        st, rg, sp = ea.el_attn_plan_preview(B, beam, heads, d_m, n, 256)
        assert st == ea.EL_OK
        return rg, sp
    # rows per workgroup in 16s, spans of the flattened tile list (workgroups = spans x row blocks)
    assert plan(64, 4, 16, 1024, 1024) == (2, 128)   # 64 rows: two blocks of 32, one workgroup per compute unit
    assert plan(320, 4, 16, 1024, 1024) == (2, 128)  # more sentences: longer spans, never more workgroups than units
    assert plan(512, 1, 16, 1024, 1024) == (1, 256)  # per-beam histories: 16 rows, one block
    assert plan(64, 4, 16, 1024, 256) == (2, 128)    # 1024 tiles: still eight per span
    assert plan(64, 4, 16, 1024, 64) == (2, 64)      # four tiles per sentence: one span per sentence, not spans of eight tiles
    assert plan(64, 4, 16, 1024, 32) == (2, 64)
    assert plan(2, 4, 16, 1024, 16) == (2, 2)        # two tiles in all
    for B in (1, 3, 17, 64, 100, 1000):
        for beam in (1, 2, 4, 5, 8):
            for n in (1, 16, 100, 1024, 4096):
                rg, sp = plan(B, beam, 16, 1024, n)
                blocks = -(-16 * beam // (16 * rg))
                assert rg == (1 if beam == 1 else 2) and 1 <= sp and sp * blocks <= max(256, blocks)
                assert sp <= B * (ea.el_attn_max_splits() - 1)             # every piece has a slot
    I = ea.EL_ERR_INVALID_ARG
    assert ea.el_attn_plan_preview(0, 4, 16, 1024, 64, 256)[0] == I
    assert ea.el_attn_plan_preview(4, 4, 16, 1024, 64, 0)[0] == I
    assert ea.el_attn_plan_preview(4, 4, 10, 640, 64, 256)[0] == ea.EL_ERR_UNSUPPORTED
    assert ea.el_attn_plan_preview(64, 4, 12, 768, 1024, 256)[:2] == (ea.EL_OK, 2)   # 48 rows: two blocks of 32


def test_check_inputs_rejects_bad_arguments_before_any_device_work(ea):
    I = ea.EL_ERR_INVALID_ARG
    A, Rp = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x20000)   # never dereferenced

    def call(dtype=ea.EL_BF16, d_model=1024, H=A, stride=64 * 1024, lengths=None, B=4, n=64, report=Rp):
        return ea.el_attn_check_inputs(dtype, d_model, H, stride, lengths, B, n, report)

    assert call(H=None) == I and call(report=None) == I
    assert call(dtype=9) == I
    for bad in (dict(d_model=0), dict(B=0), dict(n=0), dict(B=70000)):
        assert call(**bad) == I, bad
    assert call(stride=64 * 1024 - 8) == I                      # shorter than n rows
    assert call(d_model=1020) == I                              # rows not a multiple of 16 bytes
    assert call(H=ctypes.c_void_p(0x10008)) == I                # misaligned H
    assert call(report=ctypes.c_void_p(0x20004)) == I           # misaligned report


def test_build_fails_on_register_spills_in_the_attention_core():
    """The build reads hipcc's resource remarks back: spills in any instance of the core kernel are reported,
    spills elsewhere and clean instances are not."""
    from paper_2105_04779_amd import build
    core = "_ZN2el13k_core_streamILi1024ELb1ELi2ELb0EEEvNS_10StreamArgsE"
    remarks = "\n".join([
        f"core_stream.hip:95:1: remark: Function Name: {core} [-Rpass-analysis=kernel-resource-usage]",
        "core_stream.hip:95:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]",
        "core_stream.hip:95:1: remark:     VGPRs Spill: 5 [-Rpass-analysis=kernel-resource-usage]",
        "core_stream.hip:95:1: remark: Function Name: _ZN2el13k_core_streamILi512ELb0ELi1ELb0EEEvNS_10StreamArgsE [-R]",
        "core_stream.hip:95:1: remark:     VGPRs Spill: 0 [-R]",
        "gemm_mfma.hip:70:1: remark: Function Name: _ZN2el11k_gemm_slabILb1ELi1EEEvNS_8GemmArgsE [-R]",
        "gemm_mfma.hip:70:1: remark:     VGPRs Spill: 9 [-R]",
    ])
    assert build.check_core_spills(remarks) == {core: 5}
    assert build.check_core_spills("") == {}
