#!/usr/bin/env python3
"""Benchmark of the InnerQ decode-attention hot path on one MI355X.

One "step" = one decode step of one attention layer over the whole batch:
innerq_quantize_append of the new token (key evicted and quantised every step,
values spilled G at a time) followed by innerq_decode_attention over the whole
cache.  Inputs are synthetic, seeded, generated on the device, and resident in
HBM before the timed region.  Several distinct cache instances are rotated so a
timed step never re-reads bytes the previous step left in the 256 MB
last-level cache.

Prints ONE JSON line (metric / value / roofline / cpu_baseline ...).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=400)
    p.add_argument("--warmup", type=int, default=400,
                   help="untimed steps first (the device needs some 10 ms of load before its clocks settle)")
    p.add_argument("--workload", default="llama3_8b_32k")
    p.add_argument("--kind", default="inner", choices=["inner", "outer", "fp16"])
    p.add_argument("--context", type=int, default=None, metavar="N",
                   help="override the workload's context length (same shape otherwise); the result then names it")
    p.add_argument("--bits", type=int, default=None, choices=[2, 3, 4], help="code width (default: the workload's)")
    p.add_argument("--v-bits", type=int, default=0, choices=[0, 2, 3, 4],
                   help="width of the value codes when it differs from the keys' (0: the same)")
    p.add_argument("--k-mode", default=None, choices=["sym", "asym", "hybrid"])
    p.add_argument("--v-mode", default=None, choices=["sym", "asym", "hybrid"])
    p.add_argument("--instances", type=int, default=8, help="distinct caches rotated through the timed steps")
    p.add_argument("--layers", type=int, default=None, help="layers per step (default: the workload's)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--prewarm-ms", type=float, default=25.0,
                   help="untimed device pre-warm before the warm-up steps, in ms of the same work (0: none)")
    p.add_argument("--step-mode", default="fused", choices=["fused", "serial", "two-stream"],
                   help="fused (default): innerq_decode_step, i.e. attention over the cache plus the new token, then "
                        "one launch that merges the partials, appends the token and quantises one step ahead; "
                        "serial: innerq_quantize_append, then innerq_decode_attention (three launches); two-stream: "
                        "the deferred append on a side stream next to the attention")
    p.add_argument("--inner-kernel", type=int, default=0, choices=[0, 1],
                   help="0: the default fused kernel (4x4x4 fp16 matrix instructions); 1: the fp8 x fp4 "
                        "block-scaled kernel for 2-bit caches (comparison runs)")
    p.add_argument("--cpu-seconds", type=float, default=12.0)
    p.add_argument("--min-timed-ms", type=float, default=50.0,
                   help="the pass of --steps steps is repeated until the timed region is at least this long "
                        "(reported as `repeats`; 0: exactly one pass)")
    p.add_argument("--no-comparison", action="store_true",
                   help="skip the fp16 and outer-grouped comparison kernels on the same data")
    p.add_argument("--asym-frac", type=float, default=None, metavar="F",
                   help="fill the caches with crafted groups of which a fraction F is quantised asymmetrically "
                        "in hybrid mode (the rest symmetrically): the density sweep of the flag matrix "
                        "(paper, Section 'Sparsity of M')")
    p.add_argument("--sparse-zeros", action="store_true",
                   help="value zero-points are read only where a group is flagged asymmetric "
                        "(innerq_config_t.sparse_zeros = 1)")
    p.add_argument("--paged", default=None, choices=["shuffled", "identity"],
                   help="keep the quantised store in 64-row pages named by a page table (inner layout only): "
                        "shuffled = every block on a random page of the pool; identity = pages in order, which "
                        "isolates the cost of the lookup from the cost of the scatter")
    p.add_argument("--prefill", action="store_true",
                   help="time the prefill-side calls instead (key-norm calibration and the bulk append that "
                        "quantises a whole prompt) and print their rates; exits without the decode loop")
    p.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                   help="run only a plain elementwise copy of MIB mebibytes, 10 times (reference for the "
                        "rocprofv3 FETCH_SIZE / WRITE_SIZE counters), and exit")
    return p.parse_args()


PREWARM_MAX_STEPS = 1024     # cap of the device pre-warm (sizes the caches)
TIMED_MAX_STEPS = 4096       # cap of the repeated timed passes beyond the first (sizes the caches)


class Hip:
    """The handful of HIP runtime calls the benchmark makes itself (events on the launch stream)."""

    def __init__(self):
        self.rt = C.CDLL("libamdhip64.so")
        self.rt.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.rt.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.rt.hipEventDestroy.argtypes = [C.c_void_p]
        self.rt.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.rt.hipStreamWaitEvent.argtypes = [C.c_void_p, C.c_void_p, C.c_uint]

    def record(self, ev: int, stream: int) -> None:
        assert self.rt.hipEventRecord(ev, stream) == 0

    def wait(self, stream: int, ev: int) -> None:
        assert self.rt.hipStreamWaitEvent(stream, ev, 0) == 0

    def event(self) -> int:
        e = C.c_void_p()
        assert self.rt.hipEventCreate(C.byref(e)) == 0
        return e.value

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = C.c_float()
        assert self.rt.hipEventElapsedTime(C.byref(ms), a, b) == 0
        return ms.value


def algorithmic_bytes(w, cfg, iq, n_tokens, v_asym_frac=None):
    """Bytes the method itself must move per attention call over the quantised range:
    per cached (token, kv-head) K + V codes, fp16 scales and (unless symmetric) fp16 zero-points.
    A kernel that reads zero-points only for asymmetric groups (sparse_zeros) is charged the
    asymmetric fraction of the dense zero-point bytes."""
    nq_k = iq.innerq_partition(cfg, 0, n_tokens)[1]
    nq_v = iq.innerq_partition(cfg, 1, n_tokens)[1]
    n_both = min(nq_k, nq_v)
    d, b, G = w.head_dim, cfg.bits, cfg.group
    if cfg.kind == iq.KIND_FP16:
        per_unit = 2 * d * 2
    else:
        per_unit = 0
        for which, mode, bits in ((0, cfg.k_mode, cfg.bits), (1, cfg.v_mode, cfg.v_bits or cfg.bits)):
            zero_share = 0.0 if mode == iq.SYM else 1.0
            if which == 1 and cfg.sparse_zeros and cfg.kind == iq.KIND_INNER and v_asym_frac is not None:
                zero_share *= v_asym_frac
            per_unit += d * bits // 8 + (d // G) * 2 * (1 + zero_share)
    units = w.batch * w.n_kv_heads * n_both
    return per_unit, units


def crafted_groups(torch, gen, lead, G, bits, frac, device="cuda", return_mask=False):
    """Groups of G values (last axis) whose hybrid decision is known in advance: with probability
    frac a group lies exactly on an asymmetric grid of positive values (asymmetric error 0,
    symmetric error > 0), otherwise exactly on a symmetric grid (symmetric error 0; a tie goes to
    symmetric).  Every value is exact in fp16."""
    levels, den = 1 << bits, (1 << (bits - 1)) - 1
    is_asym = torch.rand(lead, device=device, generator=gen) < frac
    la = torch.randint(0, levels, (*lead, G), device=device, generator=gen)
    la[..., 0] = 0
    la[..., 1] = levels - 1
    ls = torch.randint(-den, den + 1, (*lead, G), device=device, generator=gen)
    ls[..., 0] = den
    x = torch.where(is_asym[..., None], 1.0 + 0.5 * la, 0.125 * ls).half()
    return (x, is_asym) if return_mask else x


def make_instance(torch, iq, w, cfg, layer, n_prefill, gen, asym_frac=None, shuffle_pages=True):
    """One cache filled with n_prefill synthetic tokens (values per the workload recipe, drawn on the device)."""
    B, Hk, d = w.batch, w.n_kv_heads, w.head_dim
    from paper_2602_23200_amd import workloads as wl
    sigma = torch.from_numpy(wl.key_channel_sigma(w, layer)).to("cuda", torch.float32)      # [Hk, d]
    table = None
    if cfg.page_pool_pages > 0:
        # every 64-row block of every sequence on a page of its own, the pages in random order
        table = (torch.randperm(cfg.page_pool_pages, device="cuda", generator=gen) if shuffle_pages
                 else torch.arange(cfg.page_pool_pages, device="cuda")).to(torch.int32)
        table = table.view(B, cfg.capacity_tokens // 64).contiguous()
    cache = iq.allocate_cache(cfg, page_table=table)
    if asym_frac is not None:
        G = w.group
        # keys: groups of G channels of one token; values: groups of G tokens of one channel,
        # aligned at the end of the sink window
        k = crafted_groups(torch, gen, (B, Hk, n_prefill, d // G), G, w.bits, asym_frac).reshape(B, Hk, n_prefill, d)
        n_grp = (n_prefill - w.w_sink) // G
        v = torch.randn((B, Hk, n_prefill, d), device="cuda", generator=gen).half()
        vg = crafted_groups(torch, gen, (B, Hk, n_grp, d), G, w.bits, asym_frac)          # [B, Hk, n_grp, d, G]
        v[:, :, w.w_sink:w.w_sink + n_grp * G] = vg.permute(0, 1, 2, 4, 3).reshape(B, Hk, n_grp * G, d)
        del vg
        iq.innerq_quantize_append(cache, k.contiguous(), v.contiguous())
        del k, v
        torch.cuda.synchronize()
        return cache
    k = torch.randn((B, Hk, n_prefill, d), device="cuda", generator=gen)
    k.mul_(sigma[None, :, None, :])
    k = k.half()
    v = torch.randn((B, Hk, n_prefill, d), device="cuda", generator=gen).half()
    inv = None
    if w.fold_key_norm:
        # the factors are folded into the projections at the end of prefill; the prefill keys
        # that already exist are divided on their way into the cache
        _, inv = iq.innerq_calibrate_key_norm(cfg, k, per_head=False)
    iq.innerq_quantize_append(cache, k, v, k_inv_norm=inv)
    del k, v
    torch.cuda.synchronize()
    return cache


KERNEL_SOURCES = {"inner": ["attention_inner.hip", "window_pass.h", "innerq_dev.h"],
                  "outer": ["attention_outer.hip", "window_pass.h", "innerq_dev.h"],
                  "fp16": ["attention_fp16.hip", "window_pass.h", "innerq_dev.h"]}


def kernel_sources_sha256(kind):
    """Hash of the source files of one fused attention kernel (ties a recorded profile to a build)."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES[kind]:
        h.update(open(os.path.join(ROOT, "paper_2602_23200_amd", "csrc", name), "rb").read())
    return h.hexdigest()


def compare_kinds(torch, iq, hip, w, cfg, args, gen, inner_kernel_ms, stream):
    """The comparison the paper makes (its Section "Latency": inner grouping against outer grouping and
    against an unquantised fp16 cache), on this device: the fp16 kernel and the outer-grouped kernel of
    this library over caches of the same shape, context and value distribution, their fused kernels timed
    by the same dispatch events as the inner-grouped one."""
    out = {"inner_kernel_ms": inner_kernel_ms,
           "paper_context": "the paper reports 2.7x over fp16 and 1.3x over outer grouping (KIVI-style) for its "
                            "CUDA kernels on an NVIDIA Jetson Xavier NX: other hardware, context only",
           "outer_kernel_note": "the outer-grouped kernel is built like the inner-grouped one (stored fields masked in "
                                "place as matrix operands, scales folded into the other operand once per group, "
                                "zero-point terms as per-group constants): what separates the two is what the grouping "
                                "forces (tables rebuilt per tile, the transposes)"}
    B, Hq, d = w.batch, w.n_q_heads, w.head_dim
    q = torch.randn((B, Hq, d), device="cuda", generator=gen).half()
    o = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda")
    for kind_name, kind_id in (("fp16", iq.KIND_FP16), ("outer", iq.KIND_OUTER)):
        c2 = iq.make_config(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.bits, cfg.group, cfg.w_sink,
                            cfg.w_recent, cfg.k_mode, cfg.v_mode, 0, kind_id,
                            -(-(w.n_tokens + 2 * w.group) // w.group) * w.group, cfg.v_bits)
        # enough distinct caches that a call never re-reads what the previous one left in the last-level cache
        n_inst = 3 if kind_name == "outer" else 2
        caches = [make_instance(torch, iq, w, c2, i, w.n_tokens, gen) for i in range(n_inst)]
        ws = iq.allocate_workspace(c2)
        n = 24 if kind_name == "fp16" else 48
        evs = [(hip.event(), hip.event()) for _ in range(n)]
        for i in range(n):                               # (as many untimed calls as timed ones)
            iq.innerq_decode_attention(caches[i % n_inst], q, ws, out=o, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            iq.innerq_profile_next_attention(*evs[i])
            iq.innerq_decode_attention(caches[i % n_inst], q, ws, out=o, stream=stream)
        torch.cuda.synchronize()
        call_ms = (time.perf_counter() - t0) / n * 1e3
        k_ms = sum(hip.elapsed_ms(a, b) for a, b in evs) / n
        out[f"{kind_name}_kernel_ms"] = k_ms
        out[f"{kind_name}_attention_call_ms"] = call_ms
        out[f"inner_speedup_over_{kind_name}"] = k_ms / inner_kernel_ms
        del caches, ws
        torch.cuda.empty_cache()
    return out


def prefill_rates(torch, iq, w, cfg, gen):
    """Prefill-side calls on one prompt of the workload's length: calibration reads the fp16 keys
    once; the bulk append reads fp16 keys and values once and writes the packed cache."""
    B, Hk, d, N = w.batch, w.n_kv_heads, w.head_dim, w.n_tokens
    k = torch.randn((B, Hk, N, d), device="cuda", generator=gen).half()
    v = torch.randn((B, Hk, N, d), device="cuda", generator=gen).half()
    fp16_bytes = k.numel() * 2

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    timed(lambda: iq.innerq_calibrate_key_norm(cfg, k), 2)
    t_cal = timed(lambda: iq.innerq_calibrate_key_norm(cfg, k), 10)
    caches = [iq.allocate_cache(cfg) for _ in range(3)]
    iq.innerq_quantize_append(caches[0], k, v)
    t_app = timed(lambda c=iter(caches[1:]): iq.innerq_quantize_append(next(c), k, v), 2)
    written = sum(b.numel() for b in caches[1].buffers.values() if b is not None)
    del caches
    # the two together, the keys divided by the factors on their way in: separate calls against innerq_prefill
    def separate(c):
        _, inv = iq.innerq_calibrate_key_norm(cfg, k)
        iq.innerq_quantize_append(c, k, v, k_inv_norm=inv)

    n_rep = 4
    caches = [iq.allocate_cache(cfg) for _ in range(2 * n_rep + 2)]
    separate(caches[0])
    iq.innerq_prefill(caches[1], k, v)
    t_sep = timed(lambda c=iter(caches[2:2 + n_rep]): separate(next(c)), n_rep)
    t_one = timed(lambda c=iter(caches[2 + n_rep:]): iq.innerq_prefill(next(c), k, v), n_rep)
    print(json.dumps({
        "prefill": True, "workload": w.name, "tokens": N, "batch": B,
        "calibrate_key_norm": {"ms": t_cal * 1e3, "read_GBps": fp16_bytes / t_cal / 1e9},
        "bulk_quantize_append": {"ms": t_app * 1e3, "read_GBps": 2 * fp16_bytes / t_app / 1e9,
                                 "tokens_per_s": B * N / t_app, "cache_bytes_allocated": written},
        "calibrate_then_append_with_factors": {"ms": t_sep * 1e3, "launches": 4},
        "innerq_prefill": {"ms": t_one * 1e3, "launches": 3, "tokens_per_s": B * N / t_one},
    }))


def host_cores():
    """Threads the CPU legs may use: the cores this process may run on, at most 16 (the CPU share of one
    GPU on a shared box, whatever os.cpu_count() shows there)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(n, 16))


def cpu_baseline(w, kind_id, seconds, v_bits=0):
    """The CPU oracle timed on a bounded sample of the same workload, on all host cores: whole
    (batch, kv-head) slabs, each one decode step (append one token + attention for the slab's query
    heads), one slab per thread at a time (numpy releases the interpreter lock inside its array
    operations; every thread keeps its BLAS single-threaded)."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np
    from threadpoolctl import threadpool_limits

    from oracle import innerq_oracle as orc
    from paper_2602_23200_amd import workloads as wl

    cores = host_cores()
    r = w.n_q_heads // w.n_kv_heads
    cap = -(-(w.n_tokens + 2 * w.group) // w.group) * w.group
    o = orc.Config(1, r, 1, w.head_dim, w.bits, w.group, w.w_sink, w.w_recent, w.k_mode, w.v_mode, 0,
                   kind_id, cap, v_bits)
    total_slabs = w.batch * w.n_kv_heads * w.n_layers
    per_layer = w.batch * w.n_kv_heads

    def prepare(i):
        b, h = divmod(i % per_layer, w.n_kv_heads)
        k, v = wl.kv_slab(w, b, h, n_tokens=w.n_tokens)
        cache = orc.cache_init_prefill(o, k[None, None, :-1], v[None, None, :-1])          # not timed: set-up
        return cache, k[None, None, -1], v[None, None, -1], wl.query(w)[b:b + 1, h * r:(h + 1) * r]

    def step(item):
        cache, k1, v1, q = item
        orc.append_token(o, cache, k1, v1)
        out = orc.decode_attention(o, cache, q)
        assert np.isfinite(out).all()

    done, spent, wall0 = 0, 0.0, time.perf_counter()
    with threadpool_limits(limits=1), ThreadPoolExecutor(max_workers=cores) as pool:
        # rounds of `cores` slabs: set-up in parallel (untimed), then the decode step of all of them in
        # parallel (timed, wall clock).  Bounded: stop after `seconds` of timed work or ~5x that of wall clock.
        while done < total_slabs and spent < seconds and time.perf_counter() - wall0 < 5 * seconds:
            n = min(cores, total_slabs - done)
            items = list(pool.map(prepare, range(done, done + n)))
            t0 = time.perf_counter()
            list(pool.map(step, items))
            spent += time.perf_counter() - t0
            done += n
            del items
    step_seconds = spent / done * total_slabs            # one step = every slab of every layer once
    return {"value": w.batch / step_seconds, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "host_cpu_count": os.cpu_count(),
            "sample": f"{done} of {total_slabs} (batch, kv-head) slabs of {w.name}, one decode step each "
                      f"(append + attention, {w.n_tokens} cached tokens), numpy float64, {cores} threads "
                      f"(one slab per thread; nproc = {os.cpu_count()}), {spent:.1f} s of wall clock measured, "
                      f"scaled to the full step"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    if args.copy_probe:
        n = args.copy_probe * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            torch.mul(src, 2.0, out=dst)      # one elementwise kernel: reads 4n bytes, writes 4n bytes
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe": True, "bytes_read_per_launch": 4 * n, "bytes_written_per_launch": 4 * n,
                          "launches": 10}))
        return

    from paper_2602_23200_amd import binding as iq
    from paper_2602_23200_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    w = wl.WORKLOADS[args.workload]
    if args.context is not None:
        w = w.with_(n_tokens=args.context, name=f"{w.name}@{args.context}")
    modes = {"sym": iq.SYM, "asym": iq.ASYM, "hybrid": iq.HYBRID}
    if args.bits:
        w = w.with_(bits=args.bits)
    if args.k_mode:
        w = w.with_(k_mode=modes[args.k_mode])
    if args.v_mode:
        w = w.with_(v_mode=modes[args.v_mode])
    iq.innerq_select_inner_kernel(args.inner_kernel)
    kind_id = {"inner": iq.KIND_INNER, "outer": iq.KIND_OUTER, "fp16": iq.KIND_FP16}[args.kind]
    n_layers = args.layers or w.n_layers
    K, W = args.steps, args.warmup
    # one cache per layer; single-layer workloads rotate `instances` caches instead
    n_inst = n_layers if n_layers > 1 else max(1, args.instances)
    # warm-up, pre-warm, the timed passes, the pass with events, and the breakdown passes (each at most 220 calls)
    max_steps = W + PREWARM_MAX_STEPS + (K + TIMED_MAX_STEPS) + max(K, 100) + 500
    per_inst_appends = (-(-max_steps // n_inst) + 2 if n_layers == 1 else max_steps + 2)
    cap = -(-(w.n_tokens + per_inst_appends + 2 * w.group) // 64) * 64
    if args.paged and (args.asym_frac is not None or args.sparse_zeros):
        sys.exit("bench.py: --paged is not combined with --asym-frac / --sparse-zeros")
    if args.paged and args.kind != "inner":
        sys.exit("bench.py: --paged times the inner-grouped kernel (the comparison kernels read the contiguous store only)")
    cfg = iq.make_config(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.bits, w.group, w.w_sink,
                         w.w_recent, w.k_mode, w.v_mode, 0, kind_id, cap, args.v_bits, int(args.sparse_zeros),
                         w.batch * (cap // 64) if args.paged else 0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    if args.prefill:
        prefill_rates(torch, iq, w, cfg, gen)
        return
    caches = [make_instance(torch, iq, w, cfg, i if n_layers > 1 else 0, w.n_tokens - 1, gen, args.asym_frac,
                             shuffle_pages=args.paged != "identity")
              for i in range(n_inst)]
    B, Hq, Hk, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    flag_density = None
    if (args.asym_frac is not None or args.sparse_zeros) and kind_id != iq.KIND_FP16:
        # measured share of asymmetric groups (scale sign bit) over the quantised range of cache 0
        flag_density = {}
        for which, name in ((0, "k"), (1, "v")):
            _, n_q, _ = iq.innerq_partition(cfg, which, caches[0].n_tokens)
            sc = caches[0].buffers[f"{name}_scales"].view(torch.int16)
            per_tok = d // w.group if (which == 0) == (kind_id == iq.KIND_INNER) else d
            rows = n_q if per_tok != d else n_q // w.group
            sc = sc.view(B * Hk, -1, per_tok)[:, :rows]
            flag_density[name] = float((sc < 0).float().mean().item())
    ws = iq.allocate_workspace(cfg)
    # a pool of new tokens / queries so that consecutive steps do not reuse the same inputs
    pool = 16
    k_new = torch.randn((pool, B, Hk, 1, d), device="cuda", generator=gen).half()
    v_new = torch.randn((pool, B, Hk, 1, d), device="cuda", generator=gen).half()
    q_new = torch.randn((pool, B, Hq, d), device="cuda", generator=gen).half()
    out = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    state = {"i": 0}

    def step_serial(profile=None):
        """One decode step: every layer appends its new token and attends."""
        for layer in range(n_layers):
            i = state["i"]
            state["i"] += 1
            cache = caches[i % n_inst]
            iq.innerq_quantize_append(cache, k_new[i % pool], v_new[i % pool], stream=stream)
            if profile is not None:
                iq.innerq_profile_next_attention(*profile[layer])
            iq.innerq_decode_attention(cache, q_new[i % pool], ws, out=out, stream=stream)

    hip = Hip()
    side = torch.cuda.Stream()
    main_h, side_h = stream.cuda_stream, side.cuda_stream
    ev_ready = [hip.event() for _ in range(4)]                 # inputs of a step are ready (main stream)
    ev_done = [hip.event() for _ in range(n_inst)]             # side work on cache instance j is done
    pending = [False] * n_inst

    def step_overlapped(profile=None):
        """The same work per layer, the append off the critical path: attention over the cache plus the
        new token (read from its input) on the main stream; window copy and the quantisation the next
        step needs on the side stream, ordered by events."""
        for layer in range(n_layers):
            i = state["i"]
            state["i"] += 1
            j = i % n_inst
            cache = caches[j]
            ready = ev_ready[i % 4]
            hip.record(ready, main_h)
            if pending[j]:
                hip.wait(main_h, ev_done[j])                   # this cache's previous append has finished
            if profile is not None:
                iq.innerq_profile_next_attention(*profile[layer])
            iq.innerq_decode_attention_next(cache, k_new[i % pool], v_new[i % pool], q_new[i % pool], ws, out=out,
                                            stream=stream)
            hip.wait(side_h, ready)
            iq.innerq_append_deferred(cache, k_new[i % pool], v_new[i % pool], stream=side)
            hip.record(ev_done[j], side_h)
            pending[j] = True

    def step_fused(profile=None):
        """The same work per layer in two launches: attention (new token read from its input), then
        merge + append + quantisation one step ahead."""
        for layer in range(n_layers):
            i = state["i"]
            state["i"] += 1
            if profile is not None:
                iq.innerq_profile_next_attention(*profile[layer])
            iq.innerq_decode_step(caches[i % n_inst], k_new[i % pool], v_new[i % pool], q_new[i % pool], ws, out=out,
                                  stream=stream)

    overlapped = args.step_mode != "serial"
    if overlapped:
        for cache in caches:
            iq.innerq_quantize_ahead(cache, stream=stream)
    step = {"fused": step_fused, "serial": step_serial, "two-stream": step_overlapped}[args.step_mode]

    # Device pre-warm, untimed and besides the W warm-up steps: the clocks need some 10 ms of load
    # to settle (the first passes of a cold process run 8-10 % slower), whatever W the caller picks.
    prewarm_steps = 0
    t_pw = time.perf_counter()
    while prewarm_steps < PREWARM_MAX_STEPS and (time.perf_counter() - t_pw) * 1e3 < args.prewarm_ms:
        for _ in range(8):
            step()
        prewarm_steps += 8
        torch.cuda.synchronize()
    for _ in range(W):
        step()
    torch.cuda.synchronize()
    # timed region: passes of exactly K steps, repeated (without a synchronisation in between) until the
    # region is long enough to be stable whatever K the caller picked; one host-device synchronisation
    # on either side
    repeats = 0
    t0 = time.perf_counter()
    while True:
        for _ in range(K):
            step()
        repeats += 1
        if (time.perf_counter() - t0) * 1e3 >= args.min_timed_ms or (repeats + 1) * K > K + TIMED_MAX_STEPS:
            break
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) / (K * repeats) * 1e3
    n_ctx_end = caches[0].n_tokens

    # second pass of K steps with HIP events around the dominant kernel of every attention call
    n_prof = max(K, -(-100 // n_layers))          # at least 100 dispatches, so that a small K gives a stable mean
    evs = [[(hip.event(), hip.event()) for _ in range(n_layers)] for _ in range(n_prof)]
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for s in range(n_prof):
        step(profile=evs[s])
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    durs = [hip.elapsed_ms(a, b) for per_step in evs for (a, b) in per_step]
    kern_ms = sum(durs) / len(durs)
    durs_sorted = sorted(durs)
    kern_ms_median = durs_sorted[len(durs) // 2]

    # attention-only and append-only timings (reported, not the headline)
    def time_only(fn, n):
        n = max(n, 200)                       # the closing synchronisation is amortised over enough calls
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        a = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - a) / n * 1e3

    def attn_only():
        i = state["i"]
        state["i"] += 1
        iq.innerq_decode_attention(caches[i % n_inst], q_new[i % pool], ws, out=out, stream=stream)

    def append_only():
        i = state["i"]
        state["i"] += 1
        iq.innerq_quantize_append(caches[i % n_inst], k_new[i % pool], v_new[i % pool], stream=stream)

    n_break = max(1, min(K, 400) // n_layers)
    attn_ms = time_only(attn_only, n_break * n_layers) * n_layers
    append_ms = time_only(append_only, min(n_break * n_layers, 200)) * n_layers
    # the other step mode, for the breakdown (the serial calls also work on caches that were run ahead)
    torch.cuda.synchronize()
    other_ms = time_only(step_serial, max(1, 200 // n_layers)) if overlapped else None

    per_unit, units = algorithmic_bytes(w, cfg, iq, w.n_tokens, flag_density["v"] if flag_density else None)
    alg_bytes = int(round(per_unit * units))
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9

    # yardstick: a plain streaming read of the same number of bytes (rotating buffers, so the
    # last-level cache does not help), timed the same way
    n_buf = max(2, min(8, (1 << 31) // max(alg_bytes, 1)))
    probe_bytes = (alg_bytes // 16) * 16
    bufs = [torch.empty(probe_bytes, dtype=torch.uint8, device="cuda").random_(0, 256) for _ in range(n_buf)]
    sink = torch.zeros(4, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    ev0, ev1 = evs[0][0]
    probe_ms = []
    for i in range(40):
        iq.innerq_stream_read_probe(bufs[i % n_buf], sink, ev0, ev1, stream=stream)
        torch.cuda.synchronize()
        if i >= 8:
            probe_ms.append(hip.elapsed_ms(ev0, ev1))
    del bufs
    stream_gbs = probe_bytes / (sum(probe_ms) / len(probe_ms) * 1e-3) / 1e9
    # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (a recorded figure:
    # counters cannot be read from inside this process).  The record names the kernel sources it was
    # measured with (a hash); it is reported only while those sources are unchanged, else null.
    traffic, traffic_note = None, "this workload and kernel were not profiled"
    prof_md = os.path.join(ROOT, "profiles", f"attention_{args.kind}_{w.name}_hbm_traffic.md")
    if os.path.exists(prof_md) and not (args.k_mode or args.v_mode or args.bits or args.v_bits or args.paged
                                        or args.sparse_zeros or args.asym_frac is not None):
        import re
        text = open(prof_md).read()
        m = re.search(r"^hbm_bytes_per_launch:\s*(\d+)", text, re.M)
        h = re.search(r"^kernel_sources_sha256:\s*([0-9a-f]+)", text, re.M)
        now = kernel_sources_sha256(args.kind)
        if m and h and h.group(1) == now:
            traffic, traffic_note = int(m.group(1)), f"recorded in profiles/{os.path.basename(prof_md)} for these kernel sources"
        else:
            traffic_note = (f"profiles/{os.path.basename(prof_md)} was recorded for other kernel sources "
                            f"({h.group(1)[:12] if h else 'no hash'} != {now[:12]}): not reported")

    comparison = None
    if not args.no_comparison and args.kind == "inner" and args.asym_frac is None:
        comparison = compare_kinds(torch, iq, hip, w, cfg, args, gen, kern_ms, stream)

    result = {
        "metric": "decode-attention tokens/s (one attention layer step: append of the new token with its quantisation "
                  "+ decode attention, 2-bit/4-bit inner-grouped KV) + achieved HBM GB/s of the fused kernel (% of peak)"
                  if n_layers == 1 else
                  "decode tokens/s over all layers (append with quantisation + decode attention per layer) + "
                  "achieved HBM GB/s",
        "value": B / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "repeats": repeats, "warmup": W, "prewarm_steps": prewarm_steps,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "kind": args.kind, "inner_kernel": args.inner_kernel,
                   "step_mode": args.step_mode, "batch": B, "n_q_heads": Hq, "n_kv_heads": Hk,
                   "head_dim": d, "context": w.n_tokens, "context_at_end": n_ctx_end, "bits": w.bits,
                   "v_bits": args.v_bits or w.bits,
                   "sparse_zeros": int(args.sparse_zeros), "paged_store": args.paged,
                   **({"asym_frac_requested": args.asym_frac, "asym_frac_measured": flag_density}
                      if flag_density is not None else {}),
                   "group": w.group, "w_sink": w.w_sink, "w_recent": w.w_recent,
                   "k_mode": ["sym", "asym", "hybrid"][w.k_mode], "v_mode": ["sym", "asym", "hybrid"][w.v_mode],
                   "layers": n_layers, "cache_instances": n_inst},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_note": traffic_note,
                     # the recorded HBM bytes (fetched + written, everything the launch moves: the quantised
                     # range, the fp16 windows, the queries, the split-K partials) over this run's kernel time:
                     # the rate the memory system actually sustains, next to the algorithmic one above
                     **({"traffic_GBps": traffic / (kern_ms * 1e-3) / 1e9,
                         "traffic_frac_of_peak": traffic / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "traffic_bytes_per_token_kvhead": traffic / units} if traffic else {}),
                     "kernel": "fused dequant score+value pass over the quantised range",
                     "kernel_ms_mean": kern_ms, "kernel_ms_median": kern_ms_median,
                     "algorithmic_bytes_per_launch": alg_bytes, "bytes_per_token_kvhead": per_unit,
                     "token_kvheads_per_launch": units,
                     "streaming_read_same_bytes": {"achieved": stream_gbs, "unit": "GB/s",
                                                   "frac_of_peak": stream_gbs / HBM_PEAK_GBS,
                                                   "kernel_frac_of_it": achieved / stream_gbs}},
        "breakdown_ms": {"step": ms_per_step, "step_with_events": (t3 - t2) / n_prof * 1e3,
                         "attention_only": attn_ms, "append_only": append_ms, "step_serial": other_ms},
    }
    if comparison is not None:
        result["comparison"] = comparison
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, kind_id, args.cpu_seconds, args.v_bits)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
