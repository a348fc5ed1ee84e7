"""ctypes binding of libjigsaw_decode (argument marshalling only; every step runs in the HIP kernels).

The functions carry the C ABI's names and take raw device addresses (ints).  `DecodeAttention`
is a thin convenience wrapper for PyTorch tensors: PyTorch supplies device memory and streams,
nothing else.  If the shared library is missing, loading raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libjigsaw_decode.so")

JD_OK, JD_ERR_INVALID_ARG, JD_ERR_UNSUPPORTED, JD_ERR_HIP, JD_ERR_BAD_INPUT = range(5)

# the product ABI (include/jigsaw_decode.h) and the inspection / measurement calls (include/jigsaw_decode_bench.h)
EXPORTS = ("jd_validate_config", "jd_workspace_bytes", "jd_create", "jd_decode_attention",
           "jd_decode_attention_static", "jd_append_kv",
           "jd_prefill_attention", "jd_check_device_flags", "jd_destroy", "jd_last_error_string")
BENCH_EXPORTS = ("jd_debug_partition", "jd_debug_schedule", "jd_wave_slots", "jd_debug_stream_read",
                 "jd_debug_stream_copy", "jd_bench_decode_attention_vector", "jd_bench_stream_create_cu_masked",
                 "jd_bench_stream_destroy")


class jd_config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_size", C.c_int32), ("max_pages_per_seq", C.c_int32),
                ("num_pages", C.c_int32), ("softmax_scale", C.c_float), ("cu_budget", C.c_int32)]


class JdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libjigsaw_decode status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built (python -m paper_2604_23838_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2604_23838_amd.build); "
                               "there is no fallback implementation")
        # The library and PyTorch must share one HIP runtime in the process: PyTorch brings its own copy of it,
        # and if the system's copy were loaded first (as a dependency of this library) the second one to start
        # would find no device.  With PyTorch imported first the library binds to the copy that is already there.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        l = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        l.jd_validate_config.argtypes = [C.POINTER(jd_config)]
        l.jd_validate_config.restype = C.c_int
        l.jd_workspace_bytes.argtypes = [C.POINTER(jd_config)]
        l.jd_workspace_bytes.restype = C.c_size_t
        l.jd_create.argtypes = [C.POINTER(jd_config), C.POINTER(vp)]
        l.jd_create.restype = C.c_int
        l.jd_decode_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
        l.jd_decode_attention.restype = C.c_int
        l.jd_decode_attention_static.argtypes = [C.POINTER(jd_config), vp, vp, vp, vp, vp, vp, vp]
        l.jd_decode_attention_static.restype = C.c_int
        l.jd_append_kv.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
        l.jd_append_kv.restype = C.c_int
        l.jd_prefill_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, C.c_int32, C.c_int32, vp, vp]
        l.jd_prefill_attention.restype = C.c_int
        l.jd_check_device_flags.argtypes = [vp, vp]
        l.jd_check_device_flags.restype = C.c_int
        l.jd_debug_partition.argtypes = [vp, vp, vp, vp, vp, vp]
        l.jd_debug_partition.restype = C.c_int
        l.jd_bench_decode_attention_vector.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
        l.jd_bench_decode_attention_vector.restype = C.c_int
        l.jd_bench_stream_create_cu_masked.argtypes = [C.c_int32, C.POINTER(vp)]
        l.jd_bench_stream_create_cu_masked.restype = C.c_int
        l.jd_bench_stream_destroy.argtypes = [vp]
        l.jd_bench_stream_destroy.restype = C.c_int
        l.jd_debug_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
        l.jd_debug_stream_read.restype = C.c_int
        l.jd_debug_stream_copy.argtypes = [vp, vp, C.c_size_t, vp]
        l.jd_debug_stream_copy.restype = C.c_int
        l.jd_debug_schedule.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        l.jd_debug_schedule.restype = C.c_int
        l.jd_wave_slots.argtypes = [vp]
        l.jd_wave_slots.restype = C.c_int32
        l.jd_destroy.argtypes = [vp]
        l.jd_destroy.restype = C.c_int
        l.jd_last_error_string.argtypes = [vp]
        l.jd_last_error_string.restype = C.c_char_p
        _lib = l
    return _lib


def jd_last_error_string(handle=None) -> str:
    return lib().jd_last_error_string(handle).decode()


def jd_validate_config(cfg: jd_config) -> int:
    return lib().jd_validate_config(C.byref(cfg))


def jd_workspace_bytes(cfg: jd_config) -> int:
    return int(lib().jd_workspace_bytes(C.byref(cfg)))


def jd_create(cfg: jd_config):
    h = C.c_void_p()
    st = lib().jd_create(C.byref(cfg), C.byref(h))
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(None))
    return h


def jd_decode_attention(handle, q, k_pages, v_pages, block_table, seq_lens, out, stream=0) -> None:
    """All tensor arguments are device addresses (ints); `stream` is a hipStream_t value."""
    st = lib().jd_decode_attention(handle, q, k_pages, v_pages, block_table, seq_lens, out, stream)
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(handle))


def jd_decode_attention_static(cfg: jd_config, q, k_pages, v_pages, block_table, seq_lens, out, stream=0) -> None:
    """jd_decode_attention without a handle or any allocation; device addresses (ints)."""
    st = lib().jd_decode_attention_static(C.byref(cfg), q, k_pages, v_pages, block_table, seq_lens, out, stream)
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(None))


def jd_append_kv(handle, k_new, v_new, k_pages, v_pages, block_table, seq_lens, active=None, stream=0) -> None:
    """Device addresses (ints); `active` may be None."""
    st = lib().jd_append_kv(handle, k_new, v_new, k_pages, v_pages, block_table, seq_lens, active, stream)
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(handle))


def jd_prefill_attention(handle, q, k_pages, v_pages, block_table, seq_lens, q_lens, q_offsets, total_q_rows,
                         max_q_len, out, stream=0) -> None:
    """Device addresses (ints); total_q_rows and max_q_len are host integers."""
    st = lib().jd_prefill_attention(handle, q, k_pages, v_pages, block_table, seq_lens, q_lens, q_offsets,
                                    int(total_q_rows), int(max_q_len), out, stream)
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(handle))


def jd_check_device_flags(handle, stream=0) -> None:
    st = lib().jd_check_device_flags(handle, stream)
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(handle))


def jd_debug_schedule(units: int, wave_slots: int):
    """[span, active_waves] for a work line of `units` page-units."""
    out = (C.c_int32 * 2)()
    st = lib().jd_debug_schedule(units, wave_slots, out)
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(None))
    return list(out)


def jd_wave_slots(handle) -> int:
    return int(lib().jd_wave_slots(handle))


def jd_debug_partition(handle, seq_lens, batch: int, stream=0):
    """Returns (header[8], wave_start[slots,4], cum_pages[batch+1]) as lists of ints."""
    slots = jd_wave_slots(handle)
    hdr = (C.c_int32 * 8)()
    ws = (C.c_int32 * (4 * slots))()
    cum = (C.c_int32 * (batch + 1))()
    st = lib().jd_debug_partition(handle, seq_lens, C.cast(hdr, C.c_void_p), C.cast(ws, C.c_void_p),
                                  C.cast(cum, C.c_void_p), stream)
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(handle))
    w = list(ws)
    return list(hdr), [w[4 * i:4 * i + 4] for i in range(slots)], list(cum)


def jd_bench_decode_attention_vector(handle, q, k_pages, v_pages, block_table, seq_lens, out, stream=0) -> None:
    """The decode step by the vector-ALU comparison kernels; arguments as for jd_decode_attention."""
    st = lib().jd_bench_decode_attention_vector(handle, q, k_pages, v_pages, block_table, seq_lens, out, stream)
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(handle))


def jd_bench_stream_create_cu_masked(num_cus: int) -> int:
    """A hipStream_t (as an int) confined to `num_cus` compute units."""
    h = C.c_void_p()
    st = lib().jd_bench_stream_create_cu_masked(num_cus, C.byref(h))
    if st != JD_OK:
        raise JdError(st, f"no stream confined to {num_cus} compute units")
    return int(h.value)


def jd_bench_stream_destroy(stream: int) -> None:
    st = lib().jd_bench_stream_destroy(stream)
    if st != JD_OK:
        raise JdError(st, "jd_bench_stream_destroy failed")


def jd_debug_stream_read(src, nbytes: int, sink, stream=0) -> None:
    st = lib().jd_debug_stream_read(src, nbytes, sink, stream)
    if st != JD_OK:
        raise JdError(st, "jd_debug_stream_read failed")


def jd_debug_stream_copy(dst, src, nbytes: int, stream=0) -> None:
    st = lib().jd_debug_stream_copy(dst, src, nbytes, stream)
    if st != JD_OK:
        raise JdError(st, "jd_debug_stream_copy failed")


def jd_destroy(handle) -> None:
    st = lib().jd_destroy(handle)
    if st != JD_OK:
        raise JdError(st, jd_last_error_string(None))


class DecodeAttention:
    """Handle plus tensor marshalling for PyTorch callers.

    q, k_pages, v_pages are torch.bfloat16 CUDA tensors in the library layouts
    ([B,Hq,D], [NP,Hkv,16,D]); block_table and seq_lens are int32 CUDA tensors;
    out is a float32 CUDA tensor [B,Hq,D] (allocated here when not given).
    """

    def __init__(self, batch, num_q_heads, num_kv_heads, head_dim, max_pages_per_seq, num_pages, *,
                 page_size=16, softmax_scale=0.0, cu_budget=0):
        self.cfg = jd_config(batch, num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq,
                             num_pages, softmax_scale, cu_budget)
        self.handle = jd_create(self.cfg)

    def _check(self, q, k_pages, v_pages, block_table, seq_lens, out):
        import torch
        c = self.cfg
        want = [(q, torch.bfloat16, (c.batch, c.num_q_heads, c.head_dim)),
                (k_pages, torch.bfloat16, (c.num_pages, c.num_kv_heads, c.page_size, c.head_dim)),
                (v_pages, torch.bfloat16, (c.num_pages, c.num_kv_heads, c.page_size, c.head_dim)),
                (block_table, torch.int32, (c.batch, c.max_pages_per_seq)),
                (seq_lens, torch.int32, (c.batch,)),
                (out, torch.float32, (c.batch, c.num_q_heads, c.head_dim))]
        for t, dt, shape in want:
            if not (t.is_cuda and t.dtype == dt and tuple(t.shape) == shape and t.is_contiguous()):
                raise ValueError(f"expected contiguous CUDA {dt} tensor of shape {shape}, got {t.dtype} {tuple(t.shape)}")

    def __call__(self, q, k_pages, v_pages, block_table, seq_lens, out=None, stream=None, *, vector_kernels=False):
        """One decode step.  vector_kernels=True runs the vector-ALU comparison kernels instead (benchmarks, tests)."""
        import torch
        if out is None:
            out = torch.empty((self.cfg.batch, self.cfg.num_q_heads, self.cfg.head_dim),
                              dtype=torch.float32, device=q.device)
        self._check(q, k_pages, v_pages, block_table, seq_lens, out)
        s = torch.cuda.current_stream() if stream is None else stream
        call = jd_bench_decode_attention_vector if vector_kernels else jd_decode_attention
        call(self.handle, q.data_ptr(), k_pages.data_ptr(), v_pages.data_ptr(),
             block_table.data_ptr(), seq_lens.data_ptr(), out.data_ptr(), s.cuda_stream)
        return out

    def append(self, k_new, v_new, k_pages, v_pages, block_table, seq_lens, active=None, stream=None):
        """Append one token per active request (k_new, v_new: bf16 [B, Hkv, D]) and bump seq_lens in place."""
        import torch
        c = self.cfg
        for t in (k_new, v_new):
            if not (t.is_cuda and t.dtype == torch.bfloat16 and tuple(t.shape) == (c.batch, c.num_kv_heads, c.head_dim)
                    and t.is_contiguous()):
                raise ValueError("k_new / v_new must be contiguous CUDA bf16 [B, Hkv, D]")
        if active is not None and not (active.is_cuda and active.dtype == torch.int32 and tuple(active.shape) == (c.batch,)):
            raise ValueError("active must be a CUDA int32 [B] tensor")
        s = torch.cuda.current_stream() if stream is None else stream
        jd_append_kv(self.handle, k_new.data_ptr(), v_new.data_ptr(), k_pages.data_ptr(), v_pages.data_ptr(),
                     block_table.data_ptr(), seq_lens.data_ptr(), None if active is None else active.data_ptr(),
                     s.cuda_stream)

    def prefill(self, q, k_pages, v_pages, block_table, seq_lens, q_lens, q_offsets, max_q_len, out=None, stream=None):
        """Causal attention of each request's last q_lens[b] tokens; q is bf16 [TQ, Hq, D], out fp32 [TQ, Hq, D]."""
        import torch
        c = self.cfg
        if not (q.is_cuda and q.dtype == torch.bfloat16 and q.dim() == 3 and tuple(q.shape[1:]) == (c.num_q_heads, c.head_dim)
                and q.is_contiguous()):
            raise ValueError("q must be a contiguous CUDA bf16 [TQ, Hq, D] tensor")
        for t in (q_lens, q_offsets):
            if not (t.is_cuda and t.dtype == torch.int32 and t.dim() == 1 and t.shape[0] >= c.batch):
                raise ValueError("q_lens / q_offsets must be CUDA int32 [B] tensors")
        if out is None:
            out = torch.zeros(q.shape, dtype=torch.float32, device=q.device)
        if not (out.is_cuda and out.dtype == torch.float32 and tuple(out.shape) == tuple(q.shape) and out.is_contiguous()):
            raise ValueError("out must be a contiguous CUDA float32 tensor shaped like q")
        s = torch.cuda.current_stream() if stream is None else stream
        jd_prefill_attention(self.handle, q.data_ptr(), k_pages.data_ptr(), v_pages.data_ptr(), block_table.data_ptr(),
                             seq_lens.data_ptr(), q_lens.data_ptr(), q_offsets.data_ptr(), q.shape[0], max_q_len,
                             out.data_ptr(), s.cuda_stream)
        return out

    def check_flags(self, stream=None):
        import torch
        s = torch.cuda.current_stream() if stream is None else stream
        jd_check_device_flags(self.handle, s.cuda_stream)

    def partition(self, seq_lens, stream=None):
        import torch
        s = torch.cuda.current_stream() if stream is None else stream
        return jd_debug_partition(self.handle, seq_lens.data_ptr(), self.cfg.batch, s.cuda_stream)

    def close(self):
        if self.handle is not None:
            jd_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
