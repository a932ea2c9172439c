"""ctypes binding with the same names as the C ABI (include/omniattn.h).

Argument marshalling only: every step of the decode path runs in the HIP
library.  PyTorch appears solely as the owner of device memory and streams.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libomniattn.so")
_lib = None

BF16, FP8_E4M3, FP32 = 0, 1, 2


class OmniAttnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"omniattn error {code}: {msg}")
        self.code = code


class Problem(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_heads", ctypes.c_int32), ("qk_dim", ctypes.c_int32),
        ("v_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("max_pages_per_seq", ctypes.c_int32), ("num_pages", ctypes.c_int64),
        ("sink", ctypes.c_int32), ("window", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
        ("kv_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("num_splits_hint", ctypes.c_int32), ("q_len", ctypes.c_int32),
    ]


def lib_path():
    return _LIB_PATH


def load_library():
    """Load libomniattn.so.  A library that is missing, or was not built from the present
    sources (content hash written by the build after the generated-code check has passed), is
    built first, through that check; if that is not possible the call raises.  A library
    older than its sources is never loaded."""
    global _lib
    if _lib is not None:
        return _lib
    from .build import build, is_stale
    if _LIB_PATH == os.path.join(HERE, "libomniattn.so") and is_stale():
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    P = ctypes.c_void_p
    lib.omniattn_plan.restype = ctypes.c_int
    lib.omniattn_plan.argtypes = [ctypes.POINTER(P), ctypes.POINTER(Problem), P, P]
    lib.omniattn_plan_update.restype = ctypes.c_int
    lib.omniattn_plan_update.argtypes = [P, P, P]
    lib.omniattn_plan_host.restype = ctypes.c_int
    lib.omniattn_plan_host.argtypes = [ctypes.POINTER(P), ctypes.POINTER(Problem), P, ctypes.c_int32]
    lib.omniattn_plan_destroy.restype = None
    lib.omniattn_plan_destroy.argtypes = [P]
    lib.omniattn_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.omniattn_plan_workspace_bytes.argtypes = [P]
    lib.omniattn_plan_retained_tokens.restype = ctypes.c_int64
    lib.omniattn_plan_retained_tokens.argtypes = [P]
    for name in ("num_units", "num_segments", "num_partials", "max_splits", "num_splits",
                 "tile_tokens", "head_block"):
        f = getattr(lib, "omniattn_plan_" + name)
        f.restype = ctypes.c_int32
        f.argtypes = [P]
    lib.omniattn_plan_get_segments.restype = ctypes.c_int32
    lib.omniattn_plan_get_segments.argtypes = [P, P, ctypes.c_int32]
    lib.omniattn_plan_tile_range.restype = ctypes.c_int
    lib.omniattn_plan_tile_range.argtypes = [P, ctypes.c_int32, ctypes.c_int32,
                                             ctypes.POINTER(ctypes.c_int32),
                                             ctypes.POINTER(ctypes.c_int32)]
    lib.omniattn_decode.restype = ctypes.c_int
    lib.omniattn_decode.argtypes = [P, P, P, P, P, P, P, P, ctypes.c_size_t, P]
    lib.omniattn_decode_timed.restype = ctypes.c_int
    lib.omniattn_decode_timed.argtypes = [P, P, P, P, P, P, P, P, ctypes.c_size_t, P, P, P, P]
    lib.omniattn_decode_static.restype = ctypes.c_int
    lib.omniattn_decode_static.argtypes = [P, P, P, P, P, P, P, P]
    lib.omniattn_static_scratch_bytes.restype = ctypes.c_size_t
    lib.omniattn_static_scratch_bytes.argtypes = []
    lib.omniattn_ring_pages.restype = ctypes.c_int32
    lib.omniattn_ring_pages.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.omniattn_ring_slot.restype = ctypes.c_int32
    lib.omniattn_ring_slot.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
    lib.omniattn_ring_append.restype = ctypes.c_int
    lib.omniattn_ring_append.argtypes = [ctypes.POINTER(Problem), P, P, P, P, P, P, P, P]
    lib.omniattn_strerror.restype = ctypes.c_char_p
    lib.omniattn_strerror.argtypes = [ctypes.c_int]
    lib.omniattn_last_hip_error.restype = ctypes.c_char_p
    lib.omniattn_last_hip_error.argtypes = []
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        lib = load_library()
        msg = lib.omniattn_strerror(rc).decode()
        if rc == -4:
            msg += ": " + lib.omniattn_last_hip_error().decode()
        raise OmniAttnError(rc, msg)


class Plan:
    """Owner of an omniattn_plan_t*."""

    def __init__(self, handle, problem):
        self._h = handle
        self.problem = problem
        # kept on the object: at interpreter shutdown module globals may be gone before __del__ runs
        self._destroy = load_library().omniattn_plan_destroy

    def __del__(self):
        self.destroy()

    def destroy(self):
        if getattr(self, "_h", None):
            self._destroy(self._h)
            self._h = None

    @property
    def handle(self):
        return self._h

    def _get(self, name):
        return getattr(load_library(), "omniattn_plan_" + name)(self._h)

    workspace_bytes = property(lambda self: self._get("workspace_bytes"))
    retained_tokens = property(lambda self: self._get("retained_tokens"))
    num_units = property(lambda self: self._get("num_units"))
    num_segments = property(lambda self: self._get("num_segments"))
    num_partials = property(lambda self: self._get("num_partials"))
    max_splits = property(lambda self: self._get("max_splits"))
    num_splits = property(lambda self: self._get("num_splits"))
    tile_tokens = property(lambda self: self._get("tile_tokens"))
    head_block = property(lambda self: self._get("head_block"))

    def segments(self):
        n = self.num_segments
        buf = (ctypes.c_int32 * (8 * max(n, 1)))()
        got = load_library().omniattn_plan_get_segments(self._h, buf, n)
        if got < 0:
            _check(got)
        keys = ("b", "hb", "tile_lo", "tile_hi", "slot", "unit", "L", "ntiles")
        return [dict(zip(keys, buf[8 * i:8 * i + 8])) for i in range(got)]

    def tile_range(self, b, tile):
        lo, hi = ctypes.c_int32(), ctypes.c_int32()
        _check(load_library().omniattn_plan_tile_range(self._h, b, tile, ctypes.byref(lo),
                                                       ctypes.byref(hi)))
        return lo.value, hi.value


def _problem(batch, num_heads, max_pages_per_seq, num_pages, sink, window, softmax_scale,
             kv_dtype=BF16, out_dtype=BF16, num_splits_hint=0, qk_dim=576, v_dim=512,
             page_size=128, q_len=0):
    return Problem(batch, num_heads, qk_dim, v_dim, page_size, max_pages_per_seq, num_pages,
                   sink, window, softmax_scale, kv_dtype, out_dtype, num_splits_hint, q_len)


def _lens_array(seq_lens):
    lens = [int(x) for x in seq_lens]
    return (ctypes.c_int32 * max(len(lens), 1))(*lens)


def _stream_handle(stream):
    import torch
    if stream is None:
        if not torch.cuda.is_available():
            return ctypes.c_void_p(None)  # no GPU: the library itself reports that
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def omniattn_plan(seq_lens, stream=None, **problem_fields):
    """Plan on the current HIP device; the metadata copy runs on `stream` (default: torch's
    current stream).  seq_lens: host sequence of B ints."""
    prob = _problem(**problem_fields)
    h = ctypes.c_void_p()
    _check(load_library().omniattn_plan(ctypes.byref(h), ctypes.byref(prob), _lens_array(seq_lens),
                                        _stream_handle(stream)))
    return Plan(h, prob)


def omniattn_plan_update(plan, seq_lens, stream=None):
    """Plan again for new lengths into the same object (no allocation, no synchronisation).
    seq_lens: host sequence of B ints, or a ctypes int32 array made once by the caller."""
    lens = seq_lens if isinstance(seq_lens, ctypes.Array) else _lens_array(seq_lens)
    _check(load_library().omniattn_plan_update(plan.handle, lens, _stream_handle(stream)))
    return plan


def omniattn_plan_host(seq_lens, num_cus=256, **problem_fields):
    """Host-only plan (inspection; cannot decode)."""
    prob = _problem(**problem_fields)
    h = ctypes.c_void_p()
    _check(load_library().omniattn_plan_host(ctypes.byref(h), ctypes.byref(prob),
                                             _lens_array(seq_lens), num_cus))
    return Plan(h, prob)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def omniattn_decode(plan, q, kv_cache, kv_scales, page_table, out, lse, workspace=None,
                    stream=None):
    """Launch the decode on `stream` (a torch.cuda.Stream; default: current).
    All tensors are CUDA tensors owned by the caller; nothing is allocated."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load_library().omniattn_decode(
        plan.handle, _ptr(q), _ptr(kv_cache), _ptr(kv_scales), _ptr(page_table), _ptr(out),
        _ptr(lse), _ptr(workspace), ws_bytes, ctypes.c_void_p(stream.cuda_stream)))


def omniattn_decode_timed(plan, q, kv_cache, kv_scales, page_table, out, lse, workspace, stream,
                          ev_begin, ev_main_end, ev_end):
    """omniattn_decode plus three caller-owned hipEvent_t handles (ints or None)."""
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load_library().omniattn_decode_timed(
        plan.handle, _ptr(q), _ptr(kv_cache), _ptr(kv_scales), _ptr(page_table), _ptr(out),
        _ptr(lse), _ptr(workspace), ws_bytes, ctypes.c_void_p(stream.cuda_stream),
        ev_begin, ev_main_end, ev_end))


def omniattn_decode_static(plan, q, kv_cache, kv_scales, page_table, out, lse, stream=None):
    """omniattn_decode without a workspace argument: partial rows go to the library's own
    device buffer (omniattn_static_scratch_bytes() bytes); nothing is allocated."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    _check(load_library().omniattn_decode_static(
        plan.handle, _ptr(q), _ptr(kv_cache), _ptr(kv_scales), _ptr(page_table), _ptr(out),
        _ptr(lse), ctypes.c_void_p(stream.cuda_stream)))


def omniattn_static_scratch_bytes():
    return int(load_library().omniattn_static_scratch_bytes())


def _window_union(window, q_len):
    return window + (q_len - 1 if window > 0 and q_len > 1 else 0)


def omniattn_ring_pages(sink, window, q_len=1):
    """Pages a sequence of a compressed layer owns (q_len queries per decode call)."""
    return int(load_library().omniattn_ring_pages(sink, _window_union(window, q_len)))


def omniattn_ring_slot(sink, window, logical_page, q_len=1):
    """Which of the sequence's own pages holds logical page `logical_page`."""
    return int(load_library().omniattn_ring_slot(sink, _window_union(window, q_len), logical_page))


def omniattn_ring_append(seq_lens, new_rows, new_scales, seq_pages, kv_cache, kv_scales, page_table,
                         *, sink, window, q_len=1, stream=None):
    """Append one token per sequence to a physically compressed cache (all CUDA tensors,
    seq_lens int32 [B] is incremented in place)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    fp8 = kv_cache.dtype == torch.float8_e4m3fn
    prob = _problem(batch=int(seq_lens.shape[0]), num_heads=1, max_pages_per_seq=int(page_table.shape[1]),
                    num_pages=int(kv_cache.shape[0]), sink=sink, window=window, softmax_scale=1.0,
                    kv_dtype=FP8_E4M3 if fp8 else BF16, q_len=q_len)
    _check(load_library().omniattn_ring_append(
        ctypes.byref(prob), _ptr(seq_lens), _ptr(new_rows), _ptr(new_scales), _ptr(seq_pages),
        _ptr(kv_cache), _ptr(kv_scales), _ptr(page_table), ctypes.c_void_p(stream.cuda_stream)))


def decode(q, kv_cache, kv_scales, page_table, seq_lens_host, sink, window, softmax_scale,
           out_dtype=None, num_splits_hint=0, plan=None):
    """Convenience wrapper: plan (unless given), allocate outputs/workspace with torch,
    decode.  Returns (out, lse, plan).  q [B, H, 576], or [B, T, H, 576] for T queries per
    sequence (the last T tokens, causal); out and lse are shaped alike."""
    import torch
    if not q.is_cuda:
        raise OmniAttnError(-4, "omniattn runs on the GPU only: tensors must be CUDA tensors")
    q_len = int(q.shape[1]) if q.dim() == 4 else 0
    lead = tuple(q.shape[:-1])
    B, H = int(q.shape[0]), int(q.shape[-2])
    fp8 = kv_cache.dtype == torch.float8_e4m3fn
    odt = torch.bfloat16 if out_dtype is None else out_dtype
    if plan is None:
        plan = omniattn_plan(seq_lens_host, batch=B, num_heads=H,
                             max_pages_per_seq=page_table.shape[1], num_pages=kv_cache.shape[0],
                             sink=sink, window=window, softmax_scale=softmax_scale,
                             kv_dtype=FP8_E4M3 if fp8 else BF16,
                             out_dtype=FP32 if odt == torch.float32 else BF16,
                             num_splits_hint=num_splits_hint, q_len=q_len)
    out = torch.empty(lead + (512,), dtype=odt, device=q.device)
    lse = torch.empty(lead, dtype=torch.float32, device=q.device)
    ws = None
    if plan.workspace_bytes:
        ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=q.device)
    omniattn_decode(plan, q, kv_cache, kv_scales, page_table, out, lse, ws)
    return out, lse, plan
