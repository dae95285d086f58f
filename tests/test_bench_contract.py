"""Host-only checks of bench.py's contract: it refuses more than one GPU with a message, its
workload list is the five configurations (plus the vocabulary sizes the paper selects), and its algorithmic byte / FLOP counts are the closed
forms (the head's FLOPs are the paper's 2 d k per row, Section 2.3 / Table 1)."""
import subprocess
import sys
from pathlib import Path

import bench
from paper_2603_05210_amd import synth

ROOT = Path(__file__).resolve().parent.parent


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_workloads_are_the_five_configurations():
    wl = {w["name"]: w for w in bench.workloads()}
    assert bench.workloads()[0]["name"] == "cfg2_Vd128256"    # the headline (the metric's own curve) comes first
    assert bench.workloads()[0]["H"] == 4096 and bench.workloads()[0]["rows"] == 1
    assert sorted(w["Vd"] for n, w in wl.items() if n.startswith("paper_")) == [4380, 6521, 13264]  # Sections 2.6, 3.2
    assert {n for n in wl if n.startswith("cfg1_")} == {"cfg1_B1", "cfg1_B4", "cfg1_B8"}
    assert sorted(w["Vd"] for n, w in wl.items() if n.startswith("cfg2_")) == [4096, 8192, 16384, 32768, 65536, synth.FULL_VOCAB]
    c = synth.CONFIGS
    assert (wl["cfg0"]["rows"], wl["cfg0"]["H"], wl["cfg0"]["Vd"], wl["cfg0"]["k"]) == (1, 2048, 4096, 1)
    assert (wl["cfg3"]["rows"], wl["cfg3"]["H"], wl["cfg3"]["Vd"], wl["cfg3"]["k"]) == (1024, 4096, 32000, 8)
    assert (wl["cfg4"]["rows"], wl["cfg4"]["H"], wl["cfg4"]["Vd"], wl["cfg4"]["k"]) == (512, 4096, synth.FULL_VOCAB, 16)
    assert wl["cfg4"]["peaked"] == 0.05 and len(c) == 5


def test_algorithmic_counts_are_the_closed_forms():
    w = dict(H=4096, rows=1, Vd=synth.FULL_VOCAB, k=10)
    nbytes, flops = bench.algorithmic(w)
    assert flops == 1050673152                                 # Table 1: 1050.7 M for the full head
    assert nbytes == flops + 2 * 4096 + 12 * 10                # W_sub once, h, ids + log-probs
    w = dict(H=4096, rows=1024, Vd=32000, k=8)
    nbytes, flops = bench.algorithmic(w)
    assert flops == 2 * 1024 * 4096 * 32000 and nbytes == 2 * 4096 * 32000 + 2 * 1024 * 4096 + 12 * 8 * 1024
    assert bench.HBM_PEAK_GBS == 8000.0 and bench.MFMA_BF16_PEAK_TFLOPS == 2500.0


def test_workload_description_follows_the_selected_workload():
    wl = {w["name"]: w for w in bench.workloads()}
    assert "untrimmed" in bench.describe(wl["cfg2_Vd128256"]) and "V_draft=128256" in bench.describe(wl["cfg2_Vd128256"])
    assert "untrimmed" not in bench.describe(wl["cfg2_Vd4096"]) and "V_draft=4096" in bench.describe(wl["cfg2_Vd4096"])


def test_percentile_helper():
    v = sorted(float(x) for x in range(101))
    assert bench.percentile(v, 0.5) == 50.0 and bench.percentile(v, 0.1) == 10.0 and bench.percentile(v, 0.9) == 90.0
    assert bench.percentile([], 0.5) is None and bench.percentile([3.0], 0.9) == 3.0
