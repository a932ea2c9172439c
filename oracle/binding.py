"""Build and call the C oracle (oracle/omniattn_oracle.c) through ctypes.

Test infrastructure only; see the header of the C file for what it computes
(paper section 3.2.1: attention over the sink + recent retained set).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "omniattn_oracle.c")
_LIB = os.path.join(_HERE, "libomniattn_oracle.so")
_lib = None


def lib_path():
    return _LIB


def build(force: bool = False, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the oracle with gcc (OpenMP over (b, h) pairs)."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-fno-fast-math", "-ffp-contract=off", src, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)
    return out


def _load(path=None):
    global _lib
    if path is not None:
        return _bind(ctypes.CDLL(path))
    if _lib is None:
        build()
        _lib = _bind(ctypes.CDLL(_LIB))
    return _lib


def _bind(lib):
    lib.omniattn_oracle.restype = ctypes.c_int
    lib.omniattn_oracle.argtypes = [
        ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
        ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
        ctypes.c_double, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32]
    lib.oracle_bf16_to_double.restype = ctypes.c_double
    lib.oracle_bf16_to_double.argtypes = [ctypes.c_uint16]
    lib.oracle_fp8_e4m3_to_double.restype = ctypes.c_double
    lib.oracle_fp8_e4m3_to_double.argtypes = [ctypes.c_uint8]
    lib.oracle_is_retained.restype = ctypes.c_int
    lib.oracle_is_retained.argtypes = [ctypes.c_int64] * 4
    return lib


def bf16_to_double(bits: int) -> float:
    return _load().oracle_bf16_to_double(int(bits))


def fp8_e4m3_to_double(bits: int) -> float:
    return _load().oracle_fp8_e4m3_to_double(int(bits))


def is_retained(j: int, L: int, S: int, W: int) -> bool:
    return bool(_load().oracle_is_retained(int(j), int(L), int(S), int(W)))


def _raw(t, np_dtype):
    """torch tensor (any device) or ndarray -> contiguous ndarray of raw storage words."""
    if isinstance(t, np.ndarray):
        a = t
    else:
        import torch
        t = t.detach().cpu().contiguous()
        if t.dtype == torch.bfloat16:
            t = t.view(torch.int16)
        elif t.dtype == torch.float8_e4m3fn:
            t = t.view(torch.uint8)
        a = t.numpy()
    return np.ascontiguousarray(a).view(np_dtype)


def oracle_decode(q, kv_cache, kv_scales, page_table, seq_lens, sink, window,
                  softmax_scale, *, kv_dtype="bf16", pairs=None, want_probs=False,
                  lib=None, q_len=1):
    """Run the oracle.

    q [B,H,576] bf16; kv_cache [P,128,576] bf16 or float8_e4m3fn; kv_scales
    [P,128] fp32 or None; page_table [B,max_pages] int32; seq_lens [B].
    `pairs` = optional int array [n,2] of (b, h) to evaluate (default: all).
    q_len > 1: q is [B, q_len*H', 576] (query-major), the queries are the last q_len
    tokens of each sequence and attend causally.
    The scale is first rounded to fp32, the type the decode library receives.
    Returns (out float64 [B,H,512] or [n,512], lse float64 [B,H] or [n])
    and, with want_probs, the softmax weights [.., max_L].
    """
    L = _load(lib) if isinstance(lib, str) else (lib or _load())
    B, H = int(q.shape[0]), int(q.shape[1])
    assert int(q.shape[2]) == 576
    qa = _raw(q, np.uint16)
    if kv_dtype == "bf16":
        ca, code = _raw(kv_cache, np.uint16), 0
        sa = None
    elif kv_dtype == "fp8":
        ca, code = _raw(kv_cache, np.uint8), 1
        sa = _raw(kv_scales, np.float32)
    else:
        raise ValueError(kv_dtype)
    num_pages = int(kv_cache.shape[0])
    pt = _raw(page_table, np.int32)
    max_pages = int(page_table.shape[1])
    sl = np.ascontiguousarray(np.asarray(
        seq_lens.cpu() if hasattr(seq_lens, "cpu") else seq_lens, dtype=np.int32))
    if pairs is None:
        n = B * H
        pa = None
    else:
        pa = np.ascontiguousarray(np.asarray(pairs, dtype=np.int32).reshape(-1, 2))
        n = pa.shape[0]
    out = np.empty((n, 512), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    max_L = int(sl.max()) if (want_probs and sl.size) else 0
    probs = np.empty((n, max_L), dtype=np.float64) if want_probs else None

    def p(a):
        return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None

    rc = L.omniattn_oracle(B, H, p(qa), p(ca), code, p(sa), num_pages, p(pt), max_pages,
                           p(sl), int(sink), int(window), float(np.float32(softmax_scale)), p(pa), n,
                           p(out), p(lse), p(probs), max_L, int(q_len))
    if rc != 0:
        raise RuntimeError(f"oracle failed with code {rc}")
    if pairs is None:
        out = out.reshape(B, H, 512)
        lse = lse.reshape(B, H)
        if want_probs:
            probs = probs.reshape(B, H, max_L)
    return (out, lse, probs) if want_probs else (out, lse)
