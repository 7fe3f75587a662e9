"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_per_unit_match_the_layout():
    """96 / 80 B for 2-bit G=32 (dense zero-points / symmetric only), 160 for 4-bit, 104 for the
    paper's Hybrid preset (3-bit symmetric keys, 2-bit hybrid values): the figures the roofline
    is computed from, re-derived here from the buffer sizes the library reports."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2602_23200_amd import binding as iq
    from paper_2602_23200_amd import workloads as wl
    w = wl.WORKLOADS["llama3_8b_32k"]
    cases = [((2, 0, iq.HYBRID, iq.HYBRID), 96), ((2, 0, iq.SYM, iq.SYM), 80), ((4, 0, iq.HYBRID, iq.HYBRID), 160),
             ((3, 2, iq.SYM, iq.HYBRID), 104), ((3, 0, iq.SYM, iq.SYM), 112)]
    for (bits, v_bits, km, vm), want in cases:
        cap = 4096
        cfg = iq.make_config(1, 4, 1, 128, bits, 32, 4, 128, km, vm, 0, iq.KIND_INNER, cap, v_bits)
        per_unit, units = bench.algorithmic_bytes(w, cfg, iq, 2000)
        assert per_unit == want
        # the same from the library's own buffer sizes: bytes of codes + scales + zeros per cached token
        total = sum(iq.innerq_buffer_bytes(cfg, i) for i in range(6))
        assert total == want * cap
        n_k = iq.innerq_partition(cfg, 0, 2000)[1]
        n_v = iq.innerq_partition(cfg, 1, 2000)[1]
        assert units == w.batch * w.n_kv_heads * min(n_k, n_v)
