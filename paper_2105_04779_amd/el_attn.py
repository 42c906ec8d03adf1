"""Thin Python binding of the C ABI in include/el_attn.h (argument marshalling only).

Every step of the decode path runs in the HIP library; torch is used for device
memory and the stream handle, nothing else.  Loading fails loudly when the
library has not been built -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libelattn.so")

EL_OK, EL_ERR_INVALID_ARG, EL_ERR_UNSUPPORTED, EL_ERR_ALLOC, EL_ERR_HIP, EL_ERR_WORKSPACE = range(6)
EL_F32, EL_F16, EL_BF16 = 0, 1, 2
EL_FLAG_FORCE_GENERIC = 1

DTYPE_CODES = {"f32": EL_F32, "f16": EL_F16, "bf16": EL_BF16}

EXPORTED_SYMBOLS = (
    "el_attn_prepare", "el_attn_workspace_bytes", "el_attn_bind_workspace", "el_attn_decode_step",
    "el_attn_expand_query", "el_attn_set_splits", "el_attn_max_splits", "el_attn_set_row_groups",
    "el_attn_uses_mfma", "el_attn_plan_preview", "el_attn_check_step_operands",
    "el_attn_decode_step_static",
    "el_attn_core_timing_enable", "el_attn_core_timing_read",
    "el_attn_gather_batch", "el_attn_check_inputs",
    "el_attn_decode_segment", "el_attn_merge_segments", "el_attn_max_segments",
    "el_attn_destroy", "el_attn_status_string", "el_attn_version",
)


class ElAttnConfig(ctypes.Structure):
    _fields_ = [
        ("heads", ctypes.c_int32), ("d_model", ctypes.c_int32), ("d_k", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("max_batch", ctypes.c_int32), ("max_beam", ctypes.c_int32), ("max_n", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
    ]


class ElAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2105_04779_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path.")
    # PyTorch ships a HIP runtime of its own.  The tensors this binding is handed live in that runtime, so it has to
    # be in the process before the library is loaded: loaded the other way round, the library binds to the system's
    # copy and the two runtimes then disagree about the device ("no ROCm-capable device", crashes).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.el_attn_prepare.argtypes = [ctypes.POINTER(ElAttnConfig)] + [vp] * 8 + [vp, ctypes.POINTER(vp)]
    lib.el_attn_prepare.restype = ctypes.c_int
    lib.el_attn_workspace_bytes.argtypes = [vp]
    lib.el_attn_workspace_bytes.restype = sz
    lib.el_attn_bind_workspace.argtypes = [vp, vp, sz]
    lib.el_attn_bind_workspace.restype = ctypes.c_int
    lib.el_attn_decode_step.argtypes = [vp, vp, i64, vp, vp, vp, i32, i32, i32, vp]
    lib.el_attn_decode_step.restype = ctypes.c_int
    lib.el_attn_decode_step_static.argtypes = [vp, vp, i64, vp, vp, vp, i32, i32, i32, vp]
    lib.el_attn_decode_step_static.restype = ctypes.c_int
    lib.el_attn_expand_query.argtypes = [vp, vp, vp, i32, i32, vp]
    lib.el_attn_expand_query.restype = ctypes.c_int
    lib.el_attn_set_splits.argtypes = [vp, i32]
    lib.el_attn_set_splits.restype = ctypes.c_int
    lib.el_attn_set_row_groups.argtypes = [vp, i32]
    lib.el_attn_set_row_groups.restype = ctypes.c_int
    lib.el_attn_max_splits.argtypes = []
    lib.el_attn_max_splits.restype = i32
    lib.el_attn_plan_preview.argtypes = [i32] * 6 + [ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.el_attn_plan_preview.restype = ctypes.c_int
    lib.el_attn_uses_mfma.argtypes = [vp]
    lib.el_attn_uses_mfma.restype = i32
    lib.el_attn_check_step_operands.argtypes = [ctypes.POINTER(ElAttnConfig), i32, vp, i64, vp, vp, vp, i32, i32, i32]
    lib.el_attn_check_step_operands.restype = ctypes.c_int
    lib.el_attn_core_timing_enable.argtypes = [vp, i32]
    lib.el_attn_core_timing_enable.restype = ctypes.c_int
    lib.el_attn_core_timing_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), i32, ctypes.POINTER(i32)]
    lib.el_attn_core_timing_read.restype = ctypes.c_int
    lib.el_attn_gather_batch.argtypes = [ctypes.c_int, i32, vp, i64, vp, i32, vp, i64, vp, i32, vp, i32, vp]
    lib.el_attn_gather_batch.restype = ctypes.c_int
    lib.el_attn_check_inputs.argtypes = [ctypes.c_int, i32, vp, i64, vp, i32, i32, vp, vp]
    lib.el_attn_check_inputs.restype = ctypes.c_int
    lib.el_attn_decode_segment.argtypes = [vp, vp, i64, vp, vp, vp, vp, i32, i32, i32, vp]
    lib.el_attn_decode_segment.restype = ctypes.c_int
    lib.el_attn_merge_segments.argtypes = [vp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, i32, i32, vp]
    lib.el_attn_merge_segments.restype = ctypes.c_int
    lib.el_attn_max_segments.argtypes = []
    lib.el_attn_max_segments.restype = i32
    lib.el_attn_destroy.argtypes = [vp]
    lib.el_attn_destroy.restype = ctypes.c_int
    lib.el_attn_status_string.argtypes = [ctypes.c_int]
    lib.el_attn_status_string.restype = ctypes.c_char_p
    lib.el_attn_version.argtypes = []
    lib.el_attn_version.restype = i32
    return lib


lib = _load()


# ---- functions with the C names (raw pointers as ints / None) ---------------------------------
def status_string(status: int) -> str:
    return lib.el_attn_status_string(int(status)).decode()


el_attn_status_string = status_string


def el_attn_version() -> int:
    return int(lib.el_attn_version())


def el_attn_max_splits() -> int:
    return int(lib.el_attn_max_splits())


def el_attn_prepare(cfg: ElAttnConfig, Wq, bq, Wk, bk, Wv, bv, Wo, bo, stream=None):
    """Returns (status, ctx_handle).  Pointers are device addresses (int) or None."""
    ctx = ctypes.c_void_p()
    st = lib.el_attn_prepare(ctypes.byref(cfg), Wq, bq, Wk, bk, Wv, bv, Wo, bo, stream, ctypes.byref(ctx))
    return st, ctx


def el_attn_workspace_bytes(ctx) -> int:
    return int(lib.el_attn_workspace_bytes(ctx))


def el_attn_bind_workspace(ctx, dev_ptr, nbytes) -> int:
    return lib.el_attn_bind_workspace(ctx, dev_ptr, nbytes)


def el_attn_decode_step(ctx, H, H_batch_stride, lengths, queries, out, B, beam, n, stream=None) -> int:
    return lib.el_attn_decode_step(ctx, H, H_batch_stride, lengths, queries, out, B, beam, n, stream)


def el_attn_decode_step_static(ctx, H, H_batch_stride, lengths, queries, out, B, beam, n, stream=None) -> int:
    return int(lib.el_attn_decode_step_static(ctx, H, H_batch_stride, lengths, queries, out, B, beam, n, stream))


def el_attn_expand_query(ctx, queries, elq_out, B, beam, stream=None) -> int:
    return lib.el_attn_expand_query(ctx, queries, elq_out, B, beam, stream)


def el_attn_set_splits(ctx, splits) -> int:
    return lib.el_attn_set_splits(ctx, splits)


def el_attn_set_row_groups(ctx, row_groups) -> int:
    return lib.el_attn_set_row_groups(ctx, row_groups)


def el_attn_plan_preview(B, beam, heads, d_model, n, compute_units):
    """Returns (status, row_groups, splits)."""
    rg, sp = ctypes.c_int32(0), ctypes.c_int32(0)
    st = lib.el_attn_plan_preview(B, beam, heads, d_model, n, compute_units, ctypes.byref(rg), ctypes.byref(sp))
    return st, rg.value, sp.value


def el_attn_uses_mfma(ctx) -> int:
    return int(lib.el_attn_uses_mfma(ctx))


def el_attn_check_step_operands(cfg: ElAttnConfig, mfma, H, H_batch_stride, lengths, queries, out, B, beam, n) -> int:
    return int(lib.el_attn_check_step_operands(ctypes.byref(cfg), int(mfma), H, H_batch_stride, lengths, queries, out, B, beam, n))


def el_attn_gather_batch(dtype, d_model, H_src, src_batch_stride, lengths_src, B_src,
                         H_dst, dst_batch_stride, lengths_dst, B_dst, index, n, stream=None) -> int:
    return lib.el_attn_gather_batch(dtype, d_model, H_src, src_batch_stride, lengths_src, B_src,
                                    H_dst, dst_batch_stride, lengths_dst, B_dst, index, n, stream)


def el_attn_check_inputs(dtype, d_model, H, H_batch_stride, lengths, B, n, report, stream=None) -> int:
    return lib.el_attn_check_inputs(dtype, d_model, H, H_batch_stride, lengths, B, n, report, stream)


def el_attn_decode_segment(ctx, H, H_batch_stride, lengths, queries, seg_A, seg_lse, B, beam, n, stream=None) -> int:
    return lib.el_attn_decode_segment(ctx, H, H_batch_stride, lengths, queries, seg_A, seg_lse, B, beam, n, stream)


def el_attn_merge_segments(ctx, nseg, seg_A, seg_lse, out, B, beam, stream=None) -> int:
    """seg_A, seg_lse: sequences of device addresses (int, c_void_p or None), or None."""
    def arr(ptrs):
        if ptrs is None:
            return None
        vals = [p.value if isinstance(p, ctypes.c_void_p) else p for p in ptrs]
        return (ctypes.c_void_p * max(len(vals), 1))(*vals)
    return lib.el_attn_merge_segments(ctx, nseg, arr(seg_A), arr(seg_lse), out, B, beam, stream)


def el_attn_max_segments() -> int:
    return int(lib.el_attn_max_segments())


def el_attn_core_timing_enable(ctx, max_steps) -> int:
    return lib.el_attn_core_timing_enable(ctx, max_steps)


def el_attn_core_timing_read(ctx, capacity):
    """Returns (status, [milliseconds of each recorded step's core kernel])."""
    buf = (ctypes.c_float * max(capacity, 1))()
    n = ctypes.c_int32(0)
    st = lib.el_attn_core_timing_read(ctx, buf, capacity, ctypes.byref(n))
    return st, [buf[i] for i in range(n.value)]


def el_attn_destroy(ctx) -> int:
    return lib.el_attn_destroy(ctx)


# ---- torch convenience wrapper (still marshalling only) ------------------------------------
def _torch_dtype(code):
    import torch
    return {EL_F32: torch.float32, EL_F16: torch.float16, EL_BF16: torch.bfloat16}[code]


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_handle():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def to_device(x32, dtype: str, device="cuda"):
    """float32 values already rounded to `dtype` ("f32", "f16", "bf16") -> device tensor of that dtype, bit-exact
    (argument marshalling for numpy-side callers; bf16 has no numpy type, so its bit pattern travels as int16)."""
    import numpy as np
    import torch
    from . import workloads as wl
    bits = wl.storage_bits(x32, dtype)
    if dtype == "bf16":
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(bits).to(device)


def device_weights(W: dict, dtype: str):
    """The weight dictionary of `workloads.weights` (numpy float32, rounded to `dtype`) on the device."""
    return {k: (None if v is None else to_device(v, dtype)) for k, v in W.items()}


def gather_batch(H_src, lengths_src, index, *, H_dst=None, lengths_dst=None):
    """H_dst[i, :len] = H_src[index[i], :len], lengths_dst[i] = len (marshalling only; see el_attn_gather_batch).

    H_src [B_src, n, d_m] device tensor (last two dimensions contiguous), lengths_src int32 [B_src] or None,
    index int32 [B_dst] device tensor.  Returns (H_dst, lengths_dst); fresh destination rows beyond a length
    are left as allocated.
    """
    import torch
    if H_src.dim() != 3 or H_src.stride(2) != 1 or H_src.stride(1) != H_src.shape[2]:
        raise ValueError("H_src must be [B, n, d_m] with contiguous rows")
    code = {torch.float32: EL_F32, torch.float16: EL_F16, torch.bfloat16: EL_BF16}[H_src.dtype]
    B_src, n, d_m = H_src.shape
    B_dst = int(index.shape[0])
    if index.dtype != torch.int32 or not index.is_cuda:
        raise ValueError("index must be an int32 device tensor")
    if H_dst is None:
        H_dst = torch.empty((B_dst, n, d_m), dtype=H_src.dtype, device=H_src.device)
    if lengths_dst is None and lengths_src is not None:
        lengths_dst = torch.empty((B_dst,), dtype=torch.int32, device=H_src.device)
    st = el_attn_gather_batch(code, d_m, _ptr(H_src), H_src.stride(0), _ptr(lengths_src), B_src,
                              _ptr(H_dst), H_dst.stride(0), _ptr(lengths_dst), B_dst, _ptr(index), n, _stream_handle())
    if st != EL_OK:
        raise ElAttnError(st, "el_attn_gather_batch")
    return H_dst, lengths_dst


def check_inputs(H, lengths, report=None):
    """Counts of what a decode step assumes about (H, lengths): returns a device int64 tensor
    [bad lengths, non-finite elements, elements beyond the fp16 range, elements examined] (see el_attn_check_inputs)."""
    import torch
    if H.dim() != 3 or H.stride(2) != 1 or H.stride(1) != H.shape[2]:
        raise ValueError("H must be [B, n, d_m] with contiguous rows")
    code = {torch.float32: EL_F32, torch.float16: EL_F16, torch.bfloat16: EL_BF16}[H.dtype]
    B, n, d_m = H.shape
    if lengths is not None and lengths.dtype != torch.int32:
        raise ValueError("lengths must be int32")
    if report is None:
        report = torch.empty(4, dtype=torch.int64, device=H.device)
    st = el_attn_check_inputs(code, d_m, _ptr(H), H.stride(0) if B > 1 else n * d_m, _ptr(lengths), B, n,
                              _ptr(report), _stream_handle())
    if st != EL_OK:
        raise ElAttnError(st, "el_attn_check_inputs")
    return report


class ElAttention:
    """One attention layer prepared for decode steps on the current CUDA/HIP device.

    weights: dict with Wq, Wk, Wv [d_m, h*d_k], Wo [h*d_k, d_m] and optional bq, bk, bv, bo
    as torch tensors on the device in the storage dtype.
    """

    def __init__(self, weights, *, heads, d_k, dtype, max_batch, max_beam, max_n,
                 out_dtype="f32", flags=0):
        import torch
        self._torch = torch
        d_m = weights["Wq"].shape[0]
        self.cfg = ElAttnConfig(heads, d_m, d_k, DTYPE_CODES[dtype], DTYPE_CODES[out_dtype],
                                max_batch, max_beam, max_n, flags)
        td = _torch_dtype(self.cfg.dtype)
        for k, v in weights.items():
            if v is not None:
                if not v.is_cuda or v.dtype != td or not v.is_contiguous():
                    raise ValueError(f"weight {k} must be a contiguous device tensor of dtype {td}")
        g = lambda k: _ptr(weights.get(k))
        st, ctx = el_attn_prepare(self.cfg, g("Wq"), g("bq"), g("Wk"), g("bk"), g("Wv"), g("bv"),
                                  g("Wo"), g("bo"), _stream_handle())
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_prepare")
        self.ctx = ctx
        self.d_m = d_m
        nbytes = el_attn_workspace_bytes(ctx)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=weights["Wq"].device)
        st = el_attn_bind_workspace(ctx, _ptr(self.workspace), nbytes)
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_bind_workspace")

    @property
    def uses_mfma(self) -> bool:
        return bool(el_attn_uses_mfma(self.ctx))

    def set_splits(self, splits: int):
        st = el_attn_set_splits(self.ctx, splits)
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_set_splits")

    def set_row_groups(self, row_groups: int):
        st = el_attn_set_row_groups(self.ctx, row_groups)
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_set_row_groups")

    def decode_step(self, H, lengths, queries, out=None):
        """H [B,n,d_m] (batch stride free, rows contiguous), lengths int32 [B] or None,
        queries [B,beam,d_m] contiguous.  Returns out [B,beam,d_m]."""
        torch = self._torch
        B, n, d_m = H.shape
        beam = queries.shape[1]
        if H.stride(2) != 1 or H.stride(1) != d_m:
            raise ValueError("rows of H must be contiguous with stride d_m")
        if not queries.is_contiguous():
            raise ValueError("queries must be contiguous")
        if out is None:
            out = torch.empty((B, beam, d_m), dtype=_torch_dtype(self.cfg.out_dtype), device=H.device)
        if lengths is not None and lengths.dtype != torch.int32:
            raise ValueError("lengths must be int32")
        st = el_attn_decode_step(self.ctx, _ptr(H), H.stride(0) if B > 1 else n * d_m, _ptr(lengths),
                                 _ptr(queries), _ptr(out), B, beam, n, _stream_handle())
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_decode_step")
        return out

    def decode_segment(self, H, lengths, queries):
        """a1..a6 on one key set: returns (seg_A [B*beam, h*d_k], seg_lse [B*beam, h]) in fp32."""
        torch = self._torch
        B, n, d_m = H.shape
        beam = queries.shape[1]
        if H.stride(2) != 1 or H.stride(1) != d_m:
            raise ValueError("rows of H must be contiguous with stride d_m")
        if not queries.is_contiguous():
            raise ValueError("queries must be contiguous")
        if lengths is not None and lengths.dtype != torch.int32:
            raise ValueError("lengths must be int32")
        hd = self.cfg.heads * self.cfg.d_k
        seg_A = torch.empty((B * beam, hd), dtype=torch.float32, device=H.device)
        seg_lse = torch.empty((B * beam, self.cfg.heads), dtype=torch.float32, device=H.device)
        st = el_attn_decode_segment(self.ctx, _ptr(H), H.stride(0) if B > 1 else n * d_m, _ptr(lengths),
                                    _ptr(queries), _ptr(seg_A), _ptr(seg_lse), B, beam, n, _stream_handle())
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_decode_segment")
        return seg_A, seg_lse

    def merge_segments(self, segments, B, beam, out=None):
        """segments: list of (seg_A, seg_lse) fp32 device tensors over the same B*beam rows.  Returns out [B,beam,d_m]."""
        torch = self._torch
        for A, S in segments:
            if A.dtype != torch.float32 or S.dtype != torch.float32 or not A.is_contiguous() or not S.is_contiguous():
                raise ValueError("segments must be contiguous float32 tensors")
            if A.shape[0] != B * beam or S.shape[0] != B * beam:
                raise ValueError("every segment must cover the same B*beam query rows")
        if out is None:
            out = torch.empty((B, beam, self.d_m), dtype=_torch_dtype(self.cfg.out_dtype), device=segments[0][0].device)
        st = el_attn_merge_segments(self.ctx, len(segments), [_ptr(A) for A, _ in segments],
                                    [_ptr(S) for _, S in segments], _ptr(out), B, beam, _stream_handle())
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_merge_segments")
        return out

    def core_timing(self, max_steps: int):
        st = el_attn_core_timing_enable(self.ctx, max_steps)
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_core_timing_enable")

    def read_core_timing(self, capacity: int):
        st, ms = el_attn_core_timing_read(self.ctx, capacity)
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_core_timing_read")
        return ms

    def expand_query(self, queries):
        torch = self._torch
        B, beam, d_m = queries.shape
        elq = torch.empty((B, self.cfg.heads * beam, d_m), dtype=torch.float32, device=queries.device)
        st = el_attn_expand_query(self.ctx, _ptr(queries), _ptr(elq), B, beam, _stream_handle())
        if st != EL_OK:
            raise ElAttnError(st, "el_attn_expand_query")
        return elq

    def close(self):
        if getattr(self, "ctx", None):
            el_attn_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
