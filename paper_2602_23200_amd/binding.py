"""ctypes binding of libinnerq.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; this module turns
torch tensors into device pointers, keeps the caller-owned cache buffers alive
and raises on any non-zero status.  There is no CPU fallback: if the library is
not built, importing it here fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libinnerq.so")

SYM, ASYM, HYBRID = 0, 1, 2
KIND_INNER, KIND_OUTER, KIND_FP16 = 0, 1, 2
(BUF_K_CODES, BUF_K_SCALES, BUF_K_ZEROS, BUF_V_CODES, BUF_V_SCALES, BUF_V_ZEROS,
 BUF_K_SINK, BUF_V_SINK, BUF_K_RECENT, BUF_V_RECENT, BUF_COUNT) = range(11)
BUFFER_NAMES = ("k_codes", "k_scales", "k_zeros", "v_codes", "v_scales", "v_zeros",
                "k_sink", "v_sink", "k_recent", "v_recent")

OK, E_NULL, E_ARG, E_UNSUPPORTED, E_CAPACITY, E_ALIGN, E_WORKSPACE, E_HIP = 0, -1, -2, -3, -4, -5, -6, -7


class innerq_config_t(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("bits", C.c_int32), ("group", C.c_int32),
                ("w_sink", C.c_int32), ("w_recent", C.c_int32), ("k_mode", C.c_int32),
                ("v_mode", C.c_int32), ("sym_denominator", C.c_int32), ("kind", C.c_int32),
                ("capacity_tokens", C.c_int64), ("v_bits", C.c_int32), ("sparse_zeros", C.c_int32),
                ("page_pool_pages", C.c_int64)]


class innerq_cache_t(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in BUFFER_NAMES] + [("n_tokens", C.c_int64), ("store_ahead_tokens", C.c_int64),
                                                           ("page_table", C.c_void_p)]


class InnerQError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    """Load libinnerq.so (built by __graft_entry__.build / paper_2602_23200_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2602_23200_amd.build`")
        L = C.CDLL(LIB_PATH)
        cfgp, cachep = C.POINTER(innerq_config_t), C.POINTER(innerq_cache_t)
        L.innerq_validate_config.argtypes = [cfgp]
        L.innerq_validate_config.restype = C.c_int
        L.innerq_buffer_bytes.argtypes = [cfgp, C.c_int]
        L.innerq_buffer_bytes.restype = C.c_size_t
        L.innerq_workspace_bytes.argtypes = [cfgp]
        L.innerq_workspace_bytes.restype = C.c_size_t
        L.innerq_status_string.argtypes = [C.c_int]
        L.innerq_status_string.restype = C.c_char_p
        L.innerq_partition.argtypes = [cfgp, C.c_int, C.c_int64] + [C.POINTER(C.c_int64)] * 3
        L.innerq_partition.restype = C.c_int
        L.innerq_calibrate_key_norm.argtypes = [cfgp, C.c_void_p, C.c_int64, C.c_int, C.c_void_p,
                                                C.c_void_p, C.c_void_p]
        L.innerq_calibrate_key_norm.restype = C.c_int
        L.innerq_quantize_append.argtypes = [cfgp, cachep, C.c_void_p, C.c_void_p, C.c_int64,
                                             C.c_void_p, C.c_void_p]
        L.innerq_quantize_append.restype = C.c_int
        L.innerq_prefill.argtypes = [cfgp, cachep, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p,
                                     C.c_void_p, C.c_void_p]
        L.innerq_prefill.restype = C.c_int
        L.innerq_decode_attention.argtypes = [cfgp, cachep, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                              C.c_void_p, C.c_size_t, C.c_void_p]
        L.innerq_decode_attention.restype = C.c_int
        L.innerq_decode_attention_static.argtypes = [cfgp, cachep, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                                     C.c_void_p]
        L.innerq_decode_attention_static.restype = C.c_int
        L.innerq_quantize_ahead.argtypes = [cfgp, cachep, C.c_void_p]
        L.innerq_quantize_ahead.restype = C.c_int
        L.innerq_decode_attention_next.argtypes = [cfgp, cachep, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                   C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
        L.innerq_decode_attention_next.restype = C.c_int
        L.innerq_decode_step.argtypes = [cfgp, cachep, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
        L.innerq_decode_step.restype = C.c_int
        L.innerq_decode_step_ragged.argtypes = [cfgp, cachep, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t,
                                                C.c_void_p]
        L.innerq_decode_step_ragged.restype = C.c_int
        L.innerq_append_deferred.argtypes = [cfgp, cachep, C.c_void_p, C.c_void_p, C.c_void_p]
        L.innerq_append_deferred.restype = C.c_int
        L.innerq_profile_next_attention.argtypes = [C.c_void_p, C.c_void_p]
        L.innerq_profile_next_attention.restype = C.c_int
        L.innerq_select_inner_kernel.argtypes = [C.c_int]
        L.innerq_select_inner_kernel.restype = C.c_int
        L.innerq_stream_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.innerq_stream_read_probe.restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().innerq_status_string(status).decode()


def make_config(batch, n_q_heads, n_kv_heads, head_dim, bits, group, w_sink, w_recent,
                k_mode=HYBRID, v_mode=HYBRID, sym_denominator=0, kind=KIND_INNER,
                capacity_tokens=0, v_bits=0, sparse_zeros=0, page_pool_pages=0) -> innerq_config_t:
    return innerq_config_t(batch, n_q_heads, n_kv_heads, head_dim, bits, group, w_sink, w_recent,
                           k_mode, v_mode, sym_denominator, kind, capacity_tokens, v_bits, sparse_zeros, page_pool_pages)


def innerq_validate_config(cfg: innerq_config_t) -> int:
    return lib().innerq_validate_config(C.byref(cfg))


def innerq_buffer_bytes(cfg: innerq_config_t, which: int) -> int:
    return lib().innerq_buffer_bytes(C.byref(cfg), which)


def innerq_workspace_bytes(cfg: innerq_config_t) -> int:
    return lib().innerq_workspace_bytes(C.byref(cfg))


def innerq_partition(cfg: innerq_config_t, which: int, n_tokens: int):
    a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
    st = lib().innerq_partition(C.byref(cfg), which, n_tokens, C.byref(a), C.byref(b), C.byref(c))
    if st != OK:
        raise InnerQError(st, "innerq_partition")
    return a.value, b.value, c.value


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


@dataclass
class Cache:
    """Caller-owned cache buffers (torch uint8 tensors on the GPU) plus the C struct that points at them."""
    cfg: innerq_config_t
    buffers: dict
    c: innerq_cache_t

    @property
    def n_tokens(self) -> int:
        return self.c.n_tokens

    def view(self, name: str, dtype, shape):
        return self.buffers[name].view(dtype).view(*shape)


def allocate_cache(cfg: innerq_config_t, device="cuda", page_table=None) -> Cache:
    """Allocate every buffer the configuration needs, sized by innerq_buffer_bytes, zero-filled.
    page_table: for a paged store (cfg.page_pool_pages > 0), the caller's int32 [B, capacity_tokens / 64]
    tensor on the device; the cache keeps a reference to it."""
    import torch
    st = innerq_validate_config(cfg)
    if st != OK:
        raise InnerQError(st, "allocate_cache")
    bufs, c = {}, innerq_cache_t()
    for i, name in enumerate(BUFFER_NAMES):
        n = innerq_buffer_bytes(cfg, i)
        bufs[name] = torch.zeros(n, dtype=torch.uint8, device=device) if n else None
        setattr(c, name, _ptr(bufs[name]))
    c.n_tokens = 0
    c.store_ahead_tokens = 0
    if cfg.page_pool_pages > 0:
        assert page_table is not None and page_table.dtype == torch.int32 and page_table.is_contiguous()
        assert tuple(page_table.shape) == (cfg.batch, cfg.capacity_tokens // 64)
        bufs["page_table"] = page_table
        c.page_table = _ptr(page_table)
    return Cache(cfg, bufs, c)


def allocate_workspace(cfg: innerq_config_t, device="cuda"):
    import torch
    return torch.empty(innerq_workspace_bytes(cfg), dtype=torch.uint8, device=device)


def innerq_calibrate_key_norm(cfg: innerq_config_t, k, per_head: bool = False, stream=None):
    """k: fp16 CUDA tensor [B, Hk, N, d] -> (norm, inv_norm) fp32 [Hk, d]."""
    import torch
    assert k.dtype == torch.float16 and k.is_contiguous() and k.is_cuda
    norm = torch.empty(cfg.n_kv_heads, cfg.head_dim, dtype=torch.float32, device=k.device)
    inv = torch.empty_like(norm)
    st = lib().innerq_calibrate_key_norm(C.byref(cfg), k.data_ptr(), k.shape[2], int(per_head),
                                         norm.data_ptr(), inv.data_ptr(), _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_calibrate_key_norm")
    return norm, inv


def innerq_quantize_append(cache: Cache, k_new, v_new, k_inv_norm=None, stream=None) -> None:
    """k_new, v_new: fp16 CUDA tensors [B, Hk, T, d]."""
    import torch
    for t in (k_new, v_new):
        assert t.dtype == torch.float16 and t.is_contiguous() and t.is_cuda
    assert k_new.shape == v_new.shape
    st = lib().innerq_quantize_append(C.byref(cache.cfg), C.byref(cache.c), k_new.data_ptr(), v_new.data_ptr(),
                                      k_new.shape[2], _ptr(k_inv_norm), _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_quantize_append")


def innerq_prefill(cache: Cache, k, v, per_head: bool = False, stream=None):
    """Calibrate the key factors over the prompt k and append the prompt (k divided by them) to the empty cache:
    k, v fp16 CUDA tensors [B, Hk, N, d] -> (norm, inv_norm) fp32 [Hk, d]."""
    import torch
    for t in (k, v):
        assert t.dtype == torch.float16 and t.is_contiguous() and t.is_cuda
    assert k.shape == v.shape
    norm = torch.empty(cache.cfg.n_kv_heads, cache.cfg.head_dim, dtype=torch.float32, device=k.device)
    inv = torch.empty_like(norm)
    st = lib().innerq_prefill(C.byref(cache.cfg), C.byref(cache.c), k.data_ptr(), v.data_ptr(), k.shape[2],
                              int(per_head), norm.data_ptr(), inv.data_ptr(), _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_prefill")
    return norm, inv


def innerq_decode_attention(cache: Cache, q, workspace, out=None, q_scale=None, stream=None):
    """q: fp16 CUDA tensor [B, Hq, d] -> out [B, Hq, d] (fp32 unless an fp16 `out` is passed)."""
    import torch
    assert q.dtype == torch.float16 and q.is_contiguous() and q.is_cuda
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    assert out.is_contiguous() and out.dtype in (torch.float32, torch.float16)
    st = lib().innerq_decode_attention(C.byref(cache.cfg), C.byref(cache.c), q.data_ptr(), _ptr(q_scale),
                                       out.data_ptr(), int(out.dtype == torch.float32), workspace.data_ptr(),
                                       workspace.numel() * workspace.element_size(), _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_decode_attention")
    return out


STATIC_WORKSPACE_BYTES = 32 << 20


def innerq_decode_attention_static(cache: Cache, q, out=None, q_scale=None, stream=None):
    """innerq_decode_attention with the split-K partials in the library's own static device array (no workspace)."""
    import torch
    assert q.dtype == torch.float16 and q.is_contiguous() and q.is_cuda
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    assert out.is_contiguous() and out.dtype in (torch.float32, torch.float16)
    st = lib().innerq_decode_attention_static(C.byref(cache.cfg), C.byref(cache.c), q.data_ptr(), _ptr(q_scale),
                                              out.data_ptr(), int(out.dtype == torch.float32), _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_decode_attention_static")
    return out


def innerq_quantize_ahead(cache: Cache, stream=None) -> None:
    """Writes to the store what the next single-token append will evict (n_tokens unchanged)."""
    st = lib().innerq_quantize_ahead(C.byref(cache.cfg), C.byref(cache.c), _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_quantize_ahead")


def innerq_decode_attention_next(cache: Cache, k_new, v_new, q, workspace, out=None, q_scale=None, stream=None):
    """Attention over the cache plus one token whose rows are k_new, v_new (fp16 [B, Hk, 1, d]), not yet appended."""
    import torch
    for t in (k_new, v_new, q):
        assert t.dtype == torch.float16 and t.is_contiguous() and t.is_cuda
    assert k_new.shape == v_new.shape and k_new.shape[2] == 1
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    assert out.is_contiguous() and out.dtype in (torch.float32, torch.float16)
    st = lib().innerq_decode_attention_next(C.byref(cache.cfg), C.byref(cache.c), k_new.data_ptr(), v_new.data_ptr(),
                                            q.data_ptr(), _ptr(q_scale), out.data_ptr(),
                                            int(out.dtype == torch.float32), workspace.data_ptr(),
                                            workspace.numel() * workspace.element_size(), _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_decode_attention_next")
    return out


def innerq_decode_step(cache: Cache, k_new, v_new, q, workspace, out=None, q_scale=None, stream=None):
    """innerq_decode_attention_next + innerq_append_deferred in two launches (merge and append share one)."""
    import torch
    for t in (k_new, v_new, q):
        assert t.dtype == torch.float16 and t.is_contiguous() and t.is_cuda
    assert k_new.shape == v_new.shape and k_new.shape[2] == 1
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    assert out.is_contiguous() and out.dtype in (torch.float32, torch.float16)
    st = lib().innerq_decode_step(C.byref(cache.cfg), C.byref(cache.c), k_new.data_ptr(), v_new.data_ptr(),
                                  q.data_ptr(), _ptr(q_scale), out.data_ptr(), int(out.dtype == torch.float32),
                                  workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_decode_step")
    return out


def innerq_decode_step_ragged(cache: Cache, n_tokens_dev, max_tokens: int, k_new, v_new, q, workspace, out=None,
                              q_scale=None, stream=None):
    """innerq_decode_step with one token count per sequence in device memory (int32 CUDA tensor [B], advanced by
    the call); max_tokens bounds every count + 1."""
    import torch
    for t in (k_new, v_new, q):
        assert t.dtype == torch.float16 and t.is_contiguous() and t.is_cuda
    assert n_tokens_dev.dtype == torch.int32 and n_tokens_dev.is_cuda and n_tokens_dev.is_contiguous()
    assert k_new.shape == v_new.shape and k_new.shape[2] == 1
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    st = lib().innerq_decode_step_ragged(C.byref(cache.cfg), C.byref(cache.c), n_tokens_dev.data_ptr(), max_tokens,
                                         k_new.data_ptr(), v_new.data_ptr(), q.data_ptr(), _ptr(q_scale),
                                         out.data_ptr(), int(out.dtype == torch.float32), workspace.data_ptr(),
                                         workspace.numel() * workspace.element_size(), _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_decode_step_ragged")
    return out


def sequence_view(cache: Cache, b: int) -> Cache:
    """Sequence b of a batched cache as a cache of its own (batch 1) over the same device memory: every buffer
    is laid out [B][...], so a sequence is one contiguous slice of each."""
    from dataclasses import replace as _replace
    cfg = innerq_config_t.from_buffer_copy(bytes(cache.cfg))
    assert cfg.page_pool_pages == 0, "the buffers of a paged store are pools, not per-sequence slices"
    B = cfg.batch
    cfg.batch = 1
    bufs, c = {}, innerq_cache_t()
    for name in BUFFER_NAMES:
        t = cache.buffers[name]
        bufs[name] = None if t is None else t.view(B, -1)[b]
        setattr(c, name, _ptr(bufs[name]))
    c.n_tokens = 0
    c.store_ahead_tokens = 0
    return Cache(cfg, bufs, c)


def innerq_append_deferred(cache: Cache, k_new, v_new, stream=None) -> None:
    """Copies the token k_new, v_new (fp16 [B, Hk, 1, d]) into its window and quantises one step ahead."""
    import torch
    for t in (k_new, v_new):
        assert t.dtype == torch.float16 and t.is_contiguous() and t.is_cuda
    assert k_new.shape == v_new.shape and k_new.shape[2] == 1
    st = lib().innerq_append_deferred(C.byref(cache.cfg), C.byref(cache.c), k_new.data_ptr(), v_new.data_ptr(),
                                      _stream(stream))
    if st != OK:
        raise InnerQError(st, "innerq_append_deferred")


def innerq_profile_next_attention(ev_start: Optional[int], ev_stop: Optional[int]) -> None:
    """ev_start / ev_stop: raw hipEvent_t handles (ints), or None to cancel."""
    lib().innerq_profile_next_attention(ev_start, ev_stop)


def innerq_select_inner_kernel(which: int) -> None:
    """0: 4x4x4 fp16 fused kernel everywhere (default); 1: the fp8 x fp4 kernel for 2-bit caches where it applies."""
    st = lib().innerq_select_inner_kernel(which)
    if st != OK:
        raise InnerQError(st, "innerq_select_inner_kernel")


def innerq_stream_read_probe(data, sink, ev_start: Optional[int] = None, ev_stop: Optional[int] = None,
                             stream=None) -> None:
    """Plain streaming read of the CUDA tensor `data` (byte count a multiple of 16); `sink`: >= 4 bytes."""
    st = lib().innerq_stream_read_probe(data.data_ptr(), data.numel() * data.element_size(), sink.data_ptr(),
                                        _stream(stream), ev_start, ev_stop)
    if st != OK:
        raise InnerQError(st, "innerq_stream_read_probe")
