"""The benchmark's algorithmic bytes and flops per step (what its roofline fractions divide by), checked
against the per-element figures: projection 2mn + 2mr + 4rn, Gram row 4 s rn, transform+Adam
(4 s + 18) rn, update 2mr + 2rn + 4mn bytes (bf16 gradients and weights, fp32 state), 2 m n r flop per
GEMM -- summed by hand over the 1.1B-shaped layer set."""
import bench
from paper_2410_16029_amd import workloads


def test_c5_algorithmic_bytes_and_flops():
    cfg = workloads.CONFIGS["c5"]
    mats = cfg.matrices()
    assert len(mats) == 168
    s_mn = sum(m * n for m, n in mats)
    s_rn = sum(cfg.r * n for m, n in mats)
    s_mr = sum(m * cfg.r for m, n in mats)
    assert abs(s_mn - 1207.9e6) < 0.1e6 and abs(s_rn - 260.0e6) < 0.1e6 and abs(s_mr - 218.1e6) < 0.1e6
    w = bench.algorithmic_work(cfg, mats)
    assert w["project"]["bytes"] == 2 * s_mn + 2 * s_mr + 4 * s_rn
    assert w["gram"]["bytes"] == 4 * cfg.s * s_rn
    assert w["adam"]["bytes"] == (4 * cfg.s + 18) * s_rn
    assert w["update"]["bytes"] == 2 * s_mr + 2 * s_rn + 4 * s_mn
    assert w["project"]["flops"] == w["update"]["flops"] == 2.0 * cfg.r * s_mn
    total = sum(p["bytes"] for p in w.values())
    assert abs(total / 1e9 - 47.65) < 0.01          # 5.96 ms at 8 TB/s
    # the bf16-history option halves the ring's share only
    wb = bench.algorithmic_work(cfg, mats, "bf16")
    assert wb["gram"]["bytes"] == 2 * cfg.s * s_rn and wb["adam"]["bytes"] == (2 * cfg.s + 18) * s_rn


def test_gpus_above_one_is_refused():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, bench.__file__, "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "one GPU" in res.stderr
