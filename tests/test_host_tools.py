"""Host-side pieces around the kernels that need no GPU: bench.py's command line contract and the reader that turns
rocprofv3 counter files into the per-launch traffic figures bench.py reports."""
import csv
import json
import os
import re
import subprocess
import sys

import pytest

from paper_2405_01481_amd import profile_summary as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: asked for more (by flag or by a launcher's WORLD_SIZE) bench.py says so and prints no result."""
    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "2"})):
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + argv, capture_output=True, text=True,
                           env={**os.environ, **env}, timeout=600)
        assert r.returncode != 0
        assert "ONE GPU" in r.stderr
        assert r.stdout.strip() == ""


def test_kernel_names_map_to_roofline_classes():
    """Every kernel of the hot path lands in the class bench.py prices it in: the tile kernel with the LM-head
    epilogue (5) apart from the layer GEMMs (0-4), whatever further template arguments follow."""
    want = {
        "gemm_ring_kernel<0, 2, 4, true>": "gemm_decode",
        "gemm_ring_kernel<7, 2, 4, true>": "gemm_decode",
        "attn_decode_kernel<128, 16, false, true>": "attn_decode",
        "attn_decode_kernel<64, 16, true, false>": "attn_decode",
        "gemm_dma8_kernel<3, true>": "gemm_prefill",
        "gemm_dma8_kernel<4, false>": "gemm_prefill",
        "gemm_dma8_kernel<5, true>": "lmhead_score",
        "gemm_dma_kernel<6, 128, 128, 2, 2, 2>": None,          # the exact-KL kernel is not a bench class
        "attn_prefill_kernel<128, false>": "attn_prefill",
        "resid_norm_kernel": None,
    }
    for name, cls in want.items():
        got = [c for pat, c in P.CLASSES.items() if re.match(pat, name)]
        assert got == ([cls] if cls else []), (name, got)


def _counter_csv(path, counter, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for i, (name, parts) in enumerate(rows):
            for v in parts:                      # one line per counter instance; the reader adds them up per dispatch
                w.writerow([i, name, counter, v])


def test_traffic_summary_scales_by_the_calibration_copies(tmp_path):
    """The counters are scaled by what they read for the three 1 GiB copies that come first (a counter that reads
    half the bytes of a copy doubles everything after it), summed over a dispatch's counter instances, averaged per
    class, and merged into the output file under the workload's name without touching other workloads."""
    gib = float(1 << 20)                                       # KiB
    copy = "__amd_rocclr_copyBuffer(void*, void*)"
    fetch = [(copy, [gib / 4, gib / 4])] * 3 + [(copy, [5.0])] + [
        ("void gemm_ring_kernel<0, 2, 4, true>(GemmArgs)", [1000.0, 500.0]),
        ("void gemm_ring_kernel<3, 4, 2, true>(GemmArgs)", [500.0]),
        ("void gemm_dma8_kernel<5, true>(GemmArgs)", [4000.0]),
        ("void attn_decode_kernel<128, 16, false, true>(DecodeAttnArgs)", [300.0])]
    write = [(copy, [gib])] * 3 + [
        ("void gemm_ring_kernel<0, 2, 4, true>(GemmArgs)", [100.0]),
        ("void gemm_ring_kernel<3, 4, 2, true>(GemmArgs)", [300.0]),
        ("void gemm_dma8_kernel<5, true>(GemmArgs)", [10.0]),
        ("void attn_decode_kernel<128, 16, false, true>(DecodeAttnArgs)", [1.0])]
    fcsv, wcsv, out = tmp_path / "f.csv", tmp_path / "w.csv", tmp_path / "t.json"
    _counter_csv(fcsv, "FETCH_SIZE", fetch)
    _counter_csv(wcsv, "WRITE_SIZE", write)
    out.write_text(json.dumps({"other": {"kept": 1}}))
    P.traffic(str(fcsv), str(wcsv), "8b", str(out))
    got = json.loads(out.read_text())
    assert got["other"] == {"kept": 1}
    assert got["scale_factors"]["FETCH_SIZE"] == pytest.approx(2.0) and got["scale_factors"]["WRITE_SIZE"] == pytest.approx(1.0)
    cls = got["8b"]
    dec = cls["gemm_decode"]
    assert dec["dispatches"] == 2
    assert dec["fetch_bytes_per_launch"] == pytest.approx((1500.0 + 500.0) / 2 * 2.0 * 1024)
    assert dec["write_bytes_per_launch"] == pytest.approx((100.0 + 300.0) / 2 * 1024)
    assert dec["bytes_per_launch"] == pytest.approx(dec["fetch_bytes_per_launch"] + dec["write_bytes_per_launch"])
    assert cls["lmhead_score"]["fetch_bytes_per_launch"] == pytest.approx(4000.0 * 2.0 * 1024)
    assert cls["attn_decode"]["context_dependent"] is True and dec["context_dependent"] is False
    assert "gemm_prefill" not in cls
