"""CPU-side checks of bench.py's bookkeeping: the byte and flop formulas behind the roofline figures, the committed
counter summary it quotes, and the one-GPU rule.  No GPU and no library call is needed."""
import json
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_compulsory_bytes_and_flops_of_the_production_shapes():
    """x read once, y written once, W once; the contraction on the retained modes; the pruned-transform estimate
    (the figures of the measurement plan: 537.0 MB / 4.295 G / 2.82 G for the 1-D shape, 2147.5 MB / 4.295 G / 12.1 G
    for the 2-D one)."""
    w3, w4 = bench.pick_config("cfg3"), bench.pick_config("cfg4")
    assert w3.compulsory_bytes == 8 * 256 * 1024 * (128 + 128) + 8 * 128 * 128 == 537001984
    assert w4.compulsory_bytes == 8 * 32 * 256 * 256 * (64 + 64) + 8 * 64 * 64 == 2147516416
    assert bench.flops_of(w3) == 8.0 * 256 * 128 * 128 * 128 == 4294967296.0
    assert bench.flops_of(w4) == 8.0 * 32 * 64 * 64 * 64 * 64 == 4294967296.0
    assert abs(bench.transform_flops_of(w3) / 1e9 - 2.82) < 0.01
    assert abs(bench.transform_flops_of(w4) / 1e9 - 12.1) < 0.05


def test_roofline_picks_the_larger_floor():
    """hbm when the bytes at 8 TB/s take longer than six BF16 products per multiply-add at 2.5 PFLOP/s, the matrix pipe
    otherwise, latency when both floors are below 5 us; frac is the floor over the measured time."""
    w = bench.pick_config("cfg3")
    r = bench.roofline_of(w, 100e-6)
    assert r["bound"] == "hbm" and abs(r["frac"] - 537001984 / 100e-6 / 8e12) < 1e-12
    big = bench.pick_config("cfg5_1d_B512_C256_N256_K128")
    rb = bench.roofline_of(big, 240e-6)
    assert rb["bound"] == "mfma_bf16x3"
    assert abs(rb["frac"] - bench.flops_of(big) * 6 / 2.5e15 / 240e-6) < 1e-12 and rb["frac"] > rb["hbm_frac"]
    assert bench.roofline_of(bench.pick_config("cfg1"), 6e-6)["bound"] == "latency"


def test_committed_traffic_names_kernels_that_exist():
    """profiles/traffic.json is quoted in the bench line as measured traffic: every kernel it names must still be in
    the sources, every profile it cites must exist, and the bytes must be within a few per cent of the compulsory ones
    (1-D: the spectra never leave the chip) or account for the truncated spectra (2-D)."""
    t = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    src = ""
    csrc = os.path.join(ROOT, "paper_2504_11681_amd", "csrc")
    for f in os.listdir(csrc):
        src += open(os.path.join(csrc, f)).read()
    for name, e in t.items():
        w = bench.pick_config("cfg3" if name.startswith("cfg3") else "cfg4")
        assert w.name == name
        assert os.path.exists(os.path.join(ROOT, e["source"]))
        for k in re.findall(r"k_[a-z0-9_]+", e["kernel"]):
            assert k in src, k
        ratio = e["hbm_bytes_per_launch"] / w.compulsory_bytes
        assert (1.0 <= ratio < 1.01) if w.dims == 1 else (1.10 < ratio < 1.14)


def test_more_than_one_gpu_is_refused_before_anything_runs():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
