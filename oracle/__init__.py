"""fp64 CPU oracle for the multi-head-attention decode step (TEST INFRASTRUCTURE).

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package.  It shares no code with the HIP path and never imports it.

The arithmetic lives in ``mha_oracle.c`` (plain C, double precision); this
module compiles it with gcc on first use and marshals numpy arrays to it.

``mha_reference``  multi-head attention by its definition (Eq. 1, Eq. 2/6).
``el_reference``   the same quantity in the evaluation order of Eq. 9; used by
                   the tests to check the losslessness identity on the oracle.
``segment_reference``  per-(row, head) log-sum-exp of the scores and head outputs of ordinary attention
                   over one key set, by definition (Eq. 1, Eq. 6/7), for the joint softmax of
                   section 3.2; ``join_segments_reference`` joins them and applies W^O.
``check_inputs_reference``  what a decode step assumes about its inputs, counted by definition.
``gather_batch_reference``  the state gather between decode steps (section 3.1.1's
                   state, re-ordered / compacted by the search), by its definition.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mha_oracle.c")
_LIB = os.path.join(_HERE, "libmha_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False, out: str | None = None, extra_flags=()) -> str:
    """Compile mha_oracle.c into libmha_oracle.so next to it (gcc, OpenMP).  With `out`, into that file
    instead, with `extra_flags` added (the sanitizer test builds an instrumented copy this way)."""
    lib = out or _LIB
    if force or out or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        tmp = lib + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC", *extra_flags,
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, lib)
    return lib


def _load():
    global _lib
    with _lock:
        if _lib is None:
            # MHA_ORACLE_LIB: a library built by build(out=...) to load instead (same source, other compiler flags)
            lib = ctypes.CDLL(os.environ.get("MHA_ORACLE_LIB") or build())
            dp = ctypes.POINTER(ctypes.c_double)
            ip = ctypes.POINTER(ctypes.c_int32)
            sig = [ctypes.c_int] * 6 + [dp, ip, dp] + [dp] * 8 + [dp]
            for name in ("mha_oracle", "el_oracle"):
                fn = getattr(lib, name)
                fn.argtypes = sig
                fn.restype = ctypes.c_int
            lib.oracle_num_threads.restype = ctypes.c_int
            _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the oracle's OpenMP loop over batch elements will use."""
    return int(_load().oracle_num_threads())


def _f64(a, shape, name):
    if a is None:
        return None
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if a.shape != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {a.shape}")
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _call(fn_name, H, lengths, queries, Wq, bq, Wk, bk, Wv, bv, Wo, bo, heads, d_k):
    H = np.asarray(H)
    queries = np.asarray(queries)
    if H.ndim != 3 or queries.ndim != 3:
        raise ValueError("H must be [B, n, d_m] and queries [B, beam, d_m]")
    B, n, d_m = H.shape
    beam = queries.shape[1]
    hd = heads * d_k
    H = _f64(H, (B, n, d_m), "H")
    queries = _f64(queries, (B, beam, d_m), "queries")
    Wq = _f64(Wq, (d_m, hd), "Wq")
    Wk = _f64(Wk, (d_m, hd), "Wk")
    Wv = _f64(Wv, (d_m, hd), "Wv")
    Wo = _f64(Wo, (hd, d_m), "Wo")
    bq = _f64(bq, (hd,), "bq")
    bk = _f64(bk, (hd,), "bk")
    bv = _f64(bv, (hd,), "bv")
    bo = _f64(bo, (d_m,), "bo")
    lp = None
    if lengths is not None:
        lengths = np.ascontiguousarray(np.asarray(lengths, dtype=np.int32))
        if lengths.shape != (B,):
            raise ValueError("lengths must be [B]")
        lp = lengths.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    out = np.empty((B, beam, d_m), dtype=np.float64)
    rc = getattr(_load(), fn_name)(B, beam, n, heads, d_m, d_k, _ptr(H), lp, _ptr(queries),
                                   _ptr(Wq), _ptr(bq), _ptr(Wk), _ptr(bk), _ptr(Wv), _ptr(bv),
                                   _ptr(Wo), _ptr(bo), _ptr(out))
    if rc != 0:
        raise ValueError(f"{fn_name} rejected its arguments (code {rc}); lengths must lie in [1, n]")
    return out


def mha_reference(H, lengths, queries, Wq, bq, Wk, bk, Wv, bv, Wo, bo, *, heads, d_k):
    """Eq. 6: sum_i softmax(Q_i K_i^T / sqrt(d_k)) V_i W_i^O (+ b^O), in float64.

    H [B,n,d_m]; lengths [B] or None; queries [B,beam,d_m]; Wq/Wk/Wv [d_m,h*d_k];
    Wo [h*d_k,d_m]; biases may be None.  Returns out [B,beam,d_m] float64.
    """
    return _call("mha_oracle", H, lengths, queries, Wq, bq, Wk, bk, Wv, bv, Wo, bo, heads, d_k)


def el_reference(H, lengths, queries, Wq, bq, Wk, bk, Wv, bv, Wo, bo, *, heads, d_k):
    """Eq. 9: the expanded-query evaluation order, in float64 (oracle self-check only)."""
    return _call("el_oracle", H, lengths, queries, Wq, bq, Wk, bk, Wv, bv, Wo, bo, heads, d_k)


def gather_batch_reference(H_src, lengths_src, index, H_dst_before):
    """State maintenance by its definition, one row at a time (section 3.1.1: the state is H itself).

    H_dst[i, t, :] = H_src[index[i], t, :] for t < lengths_src[index[i]]; other rows keep what
    ``H_dst_before`` held; lengths_dst[i] = lengths_src[index[i]].  An index outside [0, B_src)
    leaves its destination untouched and reports length 0.  Arrays are copied bit for bit
    (any dtype); returns (H_dst, lengths_dst).
    """
    H_src = np.asarray(H_src)
    out = np.array(H_dst_before, copy=True)
    n = H_src.shape[1]
    lens = np.full(H_src.shape[0], n, dtype=np.int32) if lengths_src is None else np.asarray(lengths_src, dtype=np.int32)
    new_lens = np.zeros(len(index), dtype=np.int32)
    for i, src in enumerate(index):
        src = int(src)
        if src < 0 or src >= H_src.shape[0]:
            continue
        new_lens[i] = lens[src]
        for t in range(int(lens[src])):
            out[i, t, :] = H_src[src, t, :]
    return out, new_lens


def segment_reference(H, lengths, queries, Wq, bq, Wk, bk, Wv, bv, *, heads, d_k):
    """Ordinary attention over one key set, left unjoined (section 3.2 combines such pieces under one softmax).

    Per query row m = b*beam + j and head i, with K_i = H_b W_i^K + b_i^K, V_i = H_b W_i^V + b_i^V (Eq. 6) and
    s_t = Q_i K_i[t]^T / sqrt(d_k) for t < lengths[b] (Eq. 1):
        lse[m, i] = log sum_t exp(s_t)            seg_A[m, i*d_k:(i+1)*d_k] = softmax(s) V_i
    Everything in float64; returns (seg_A [B*beam, h*d_k], lse [B*beam, h]).
    """
    H = np.asarray(H, dtype=np.float64)
    q = np.asarray(queries, dtype=np.float64)
    B, n, d_m = H.shape
    beam = q.shape[1]
    hd = heads * d_k
    zeros = np.zeros(hd)
    bq, bk, bv = [zeros if b is None else np.asarray(b, dtype=np.float64) for b in (bq, bk, bv)]
    Wq, Wk, Wv = [np.asarray(W, dtype=np.float64) for W in (Wq, Wk, Wv)]
    lens = np.full(B, n, dtype=np.int64) if lengths is None else np.asarray(lengths, dtype=np.int64)
    seg_A = np.zeros((B * beam, hd))
    lse = np.zeros((B * beam, heads))
    for b in range(B):
        Hb = H[b, :lens[b]]
        K = Hb @ Wk + bk
        V = Hb @ Wv + bv
        for j in range(beam):
            Q = q[b, j] @ Wq + bq
            for i in range(heads):
                cols = slice(i * d_k, (i + 1) * d_k)
                s = K[:, cols] @ Q[cols] / np.sqrt(d_k)
                m = s.max()
                e = np.exp(s - m)
                lse[b * beam + j, i] = m + np.log(e.sum())
                seg_A[b * beam + j, cols] = (e / e.sum()) @ V[:, cols]
    return seg_A, lse


def join_segments_reference(segments, Wo, bo, *, heads, d_k):
    """One softmax over the union of the segments' keys, then Eq. 2's output projection.

    segments: list of (seg_A, lse) as segment_reference returns them, all over the same query rows.
    A softmax over a union of key sets is the mixture of the per-set softmaxes with weights
    proportional to each set's sum of exponentials, exp(lse_s).  Returns out [rows, d_m] float64.
    """
    Wo = np.asarray(Wo, dtype=np.float64)
    rows = segments[0][0].shape[0]
    A = np.zeros((rows, heads * d_k))
    for r in range(rows):
        for i in range(heads):
            cols = slice(i * d_k, (i + 1) * d_k)
            M = max(l[r, i] for _, l in segments)
            w = np.array([np.exp(l[r, i] - M) for _, l in segments])
            w /= w.sum()
            for (sA, _), ws in zip(segments, w):
                A[r, cols] += ws * sA[r, cols]
    out = A @ Wo
    if bo is not None:
        out = out + np.asarray(bo, dtype=np.float64)
    return out


def check_inputs_reference(H, lengths, n=None):
    """Counts of what the decode step assumes about its inputs (section 3.1 needs a non-empty softmax; the 16-bit
    path needs fp16-representable magnitudes), one element at a time over the valid rows only.

    H [B, n, d_m] as float32/float64 VALUES of the stored elements (NaN/Inf allowed); lengths [B] or None.
    Returns [lengths outside [1, n], non-finite elements, finite elements with |v| > 65504, elements examined];
    a length outside [0, n] is clamped for the walk.
    """
    H = np.asarray(H)
    B, n_rows, d_m = H.shape
    n = n_rows if n is None else n
    lens = np.full(B, n, dtype=np.int64) if lengths is None else np.asarray(lengths, dtype=np.int64)
    bad_len = nonfinite = large = seen = 0
    for b in range(B):
        if lens[b] < 1 or lens[b] > n:
            bad_len += 1
        for t in range(int(min(max(lens[b], 0), n))):
            row = H[b, t].astype(np.float64)
            fin = np.isfinite(row)
            nonfinite += int((~fin).sum())
            large += int((np.abs(row[fin]) > 65504.0).sum())
            seen += d_m
    return [bad_len, nonfinite, large, seen]
