"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol include/innerq.h declares, validates arguments before touching the device, and
its size / partition arithmetic agrees with the oracle's independent one."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import innerq_oracle as orc
from paper_2602_23200_amd import binding as iq
from paper_2602_23200_amd import workloads as wl
from tests.helpers import oracle_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "innerq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(innerq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"innerq_calibrate_key_norm", "innerq_quantize_append", "innerq_decode_attention",
            "innerq_buffer_bytes", "innerq_workspace_bytes", "innerq_status_string",
            "innerq_validate_config", "innerq_partition"} <= set(names)
    L = iq.lib()
    for n in names:
        assert getattr(L, n) is not None


def cfg_of(w, kind=iq.KIND_INNER, **over):
    o = oracle_config(w, kind=kind)
    c = iq.make_config(o.batch, o.n_q_heads, o.n_kv_heads, o.head_dim, o.bits, o.group, o.w_sink,
                       o.w_recent, o.k_mode, o.v_mode, o.sym_denominator, kind, o.capacity_tokens)
    for k, v in over.items():
        setattr(c, k, v)
    return c, o


def test_struct_layout_matches_header_order():
    # twelve int32, one int64, one int32 (+ tail padding to the int64 alignment)
    assert C.sizeof(iq.innerq_config_t) == 12 * 4 + 8 + 8 + 8
    assert iq.innerq_config_t.capacity_tokens.offset == 48 and iq.innerq_config_t.v_bits.offset == 56
    assert iq.innerq_config_t.sparse_zeros.offset == 60 and iq.innerq_config_t.page_pool_pages.offset == 64
    assert C.sizeof(iq.innerq_cache_t) == 10 * 8 + 8 + 8 + 8
    assert iq.innerq_cache_t.store_ahead_tokens.offset == 88 and iq.innerq_cache_t.page_table.offset == 96


def test_validate_config_rejections():
    w = wl.WORKLOADS["tiny"]
    good, _ = cfg_of(w)
    assert iq.innerq_validate_config(good) == iq.OK
    cases = [
        (dict(n_q_heads=6, n_kv_heads=4), iq.E_ARG),
        (dict(group=48), iq.E_ARG),                  # does not tile head_dim
        (dict(group=16), iq.E_UNSUPPORTED),
        (dict(bits=5), iq.E_UNSUPPORTED),            # only 2, 3 and 4 bits are built
        (dict(bits=8), iq.E_UNSUPPORTED),
        (dict(bits=0), iq.E_ARG),
        (dict(v_bits=5), iq.E_UNSUPPORTED),
        (dict(v_bits=-1), iq.E_ARG),
        (dict(head_dim=64, group=32), iq.E_UNSUPPORTED),
        (dict(w_recent=0), iq.E_ARG),
        (dict(w_sink=-1), iq.E_ARG),
        (dict(k_mode=3), iq.E_ARG),
        (dict(kind=5), iq.E_ARG),
        (dict(sym_denominator=2), iq.E_ARG),
        (dict(capacity_tokens=100), iq.E_ARG),       # not a multiple of the group
        (dict(batch=0), iq.E_ARG),
    ]
    for over, want in cases:
        bad, _ = cfg_of(w, **over)
        assert iq.innerq_validate_config(bad) == want, over
        assert iq.innerq_buffer_bytes(bad, iq.BUF_K_CODES) == 0
        assert iq.innerq_workspace_bytes(bad) == 0
    assert "not supported" in iq.status_string(iq.E_UNSUPPORTED)
    assert iq.status_string(0) == "ok"


@pytest.mark.parametrize("kind", [iq.KIND_INNER, iq.KIND_OUTER, iq.KIND_FP16])
@pytest.mark.parametrize("name", ["tiny", "llama3_8b_32k", "mistral_7b_8k"])
def test_buffer_bytes_match_oracle_buffers(kind, name):
    w = wl.WORKLOADS[name].with_(batch=1, n_tokens=512)
    for mode, bits, v_bits in ((iq.SYM, w.bits, 0), (iq.HYBRID, w.bits, 0), (iq.HYBRID, 3, 0), (iq.SYM, 3, 2),
                               (iq.HYBRID, 2, 4)):
        c, o = cfg_of(w.with_(k_mode=mode, v_mode=mode, bits=bits), kind=kind, v_bits=v_bits)
        o.v_bits = v_bits
        cache = orc.cache_new(o)
        for i, f in enumerate(iq.BUFFER_NAMES):
            a = getattr(cache, f)
            want = 0 if a is None else a.nbytes
            if f.endswith("zeros") and mode == iq.SYM:
                want = 0                              # symmetric tensors store no zero-points
            assert iq.innerq_buffer_bytes(c, i) == want, f
        assert iq.innerq_workspace_bytes(c) > 0


@pytest.mark.parametrize("kind", [iq.KIND_INNER, iq.KIND_OUTER, iq.KIND_FP16])
def test_partition_matches_oracle(kind):
    w = wl.WORKLOADS["mistral_7b_8k"]
    c, o = cfg_of(w, kind=kind)
    for n in list(range(0, 400)) + [8191, 8192, 8193]:
        for which, x in ((0, "k"), (1, "v")):
            assert iq.innerq_partition(c, which, n) == orc.partition(o, x, n)


def test_calls_reject_bad_arguments_before_any_launch():
    """All of these must fail on the host (no GPU here): status < 0, counter untouched."""
    w = wl.WORKLOADS["tiny"]
    c, _ = cfg_of(w)
    L = iq.lib()
    cache = iq.innerq_cache_t()
    # null buffers
    assert L.innerq_quantize_append(C.byref(c), C.byref(cache), 16, 16, 1, None, None) == iq.E_NULL
    assert L.innerq_decode_attention(C.byref(c), C.byref(cache), 16, None, 16, 1, 16, 1 << 30, None) == iq.E_NULL
    assert L.innerq_calibrate_key_norm(C.byref(c), None, 4, 0, 16, 16, None) == iq.E_NULL
    # fake but aligned pointers: argument errors are still caught first
    for n in iq.BUFFER_NAMES:
        setattr(cache, n, 4096)
    assert L.innerq_quantize_append(C.byref(c), C.byref(cache), 4096, 4096, -1, None, None) == iq.E_ARG
    cache.n_tokens = c.capacity_tokens
    assert L.innerq_quantize_append(C.byref(c), C.byref(cache), 4096, 4096, 1, None, None) == iq.E_CAPACITY
    assert cache.n_tokens == c.capacity_tokens
    cache.n_tokens = 10
    assert L.innerq_quantize_append(C.byref(c), C.byref(cache), 4097, 4096, 1, None, None) == iq.E_ALIGN
    assert L.innerq_decode_attention(C.byref(c), C.byref(cache), 4096, None, 4096, 1, 4096, 8, None) == iq.E_WORKSPACE
    assert L.innerq_decode_attention(C.byref(c), C.byref(cache), 4098, None, 4096, 1, 4096, 1 << 30, None) == iq.E_ALIGN
    # the one-step-ahead calls refuse a cache whose store was not run ahead (nothing records it otherwise,
    # and the kernels would read store rows that were never written)
    cache.store_ahead_tokens = 10
    assert L.innerq_decode_attention_next(C.byref(c), C.byref(cache), 4096, 4096, 4096, None, 4096, 1, 4096,
                                          1 << 30, None) == iq.E_ARG
    assert L.innerq_decode_step(C.byref(c), C.byref(cache), 4096, 4096, 4096, None, 4096, 1, 4096, 1 << 30,
                                None) == iq.E_ARG
    assert cache.n_tokens == 10 and cache.store_ahead_tokens == 10
    cache.n_tokens = 0
    assert L.innerq_decode_attention(C.byref(c), C.byref(cache), 4096, None, 4096, 1, 4096, 1 << 30, None) == iq.E_ARG
    cache.k_scales = 4104
    assert L.innerq_quantize_append(C.byref(c), C.byref(cache), 4096, 4096, 1, None, None) == iq.E_ALIGN
    assert L.innerq_calibrate_key_norm(C.byref(c), 4096, 0, 0, 4096, 4096, None) == iq.E_ARG
    bad, _ = cfg_of(w, bits=5)
    assert L.innerq_quantize_append(C.byref(bad), C.byref(cache), 4096, 4096, 1, None, None) == iq.E_UNSUPPORTED


def test_static_workspace_entry_rejects_what_does_not_fit():
    """The size check comes before any device call, so it can be exercised without a GPU."""
    L = iq.lib()
    # 512 sequences x 32 query heads need more partial slots than the static array holds
    cfg = iq.make_config(512, 32, 8, 128, 2, 32, 4, 128, capacity_tokens=256)
    assert iq.innerq_workspace_bytes(cfg) > iq.STATIC_WORKSPACE_BYTES
    cache = iq.innerq_cache_t()
    for n in iq.BUFFER_NAMES:
        setattr(cache, n, 4096)
    cache.n_tokens = 8
    assert L.innerq_decode_attention_static(C.byref(cfg), C.byref(cache), 4096, None, 4096, 1, None) == iq.E_WORKSPACE
    header = open(os.path.join(ROOT, "include", "innerq.h")).read()
    assert f"INNERQ_STATIC_WORKSPACE_BYTES ({iq.STATIC_WORKSPACE_BYTES >> 20}u << 20)" in header


def test_paged_store_sizes_and_rejections():
    """A paged store: the six store buffers are sized by the pool, the windows by the batch; the page table
    is required and checked on the host."""
    w = wl.WORKLOADS["tiny"]
    c, o = cfg_of(w, capacity_tokens=1280)
    store = ("k_codes", "k_scales", "k_zeros", "v_codes", "v_scales", "v_zeros")
    flat = [iq.innerq_buffer_bytes(c, i) for i in range(len(iq.BUFFER_NAMES))]
    c.page_pool_pages = 7
    assert iq.innerq_validate_config(c) == iq.OK
    paged = [iq.innerq_buffer_bytes(c, i) for i in range(len(iq.BUFFER_NAMES))]
    for i, name in enumerate(iq.BUFFER_NAMES):
        if name in store:
            assert paged[i] * c.batch * (c.capacity_tokens // 64) == flat[i] * 7, name
        else:
            assert paged[i] == flat[i], name
    L = iq.lib()
    cache = iq.innerq_cache_t()
    for n in iq.BUFFER_NAMES:
        setattr(cache, n, 4096)
    cache.n_tokens = 10
    assert L.innerq_quantize_append(C.byref(c), C.byref(cache), 4096, 4096, 1, None, None) == iq.E_NULL
    cache.page_table = 4098
    assert L.innerq_decode_attention(C.byref(c), C.byref(cache), 4096, None, 4096, 1, 4096, 1 << 30, None) == iq.E_ALIGN
    c.page_pool_pages = -1
    assert iq.innerq_validate_config(c) == iq.E_ARG
    c.page_pool_pages = 7
    c.capacity_tokens = 1280 + 32                                   # not a whole number of pages
    assert iq.innerq_validate_config(c) == iq.E_ARG
