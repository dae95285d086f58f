#!/usr/bin/env python3
"""Benchmark of the trimmed-vocabulary draft LM head on one MI355X.

A "step" is one draft step through the C ABI: vt_draft_head (projection over the draft
vocabulary with fused softmax statistics and top-k, merge, d2t remap) on inputs already in
HBM.  vt_build_subset is the one-time set-up per draft vocabulary (Section 2.1 of the paper)
and is timed separately ("build_subset" in the output), not as part of a step.

Headline workload: the untrimmed baseline head at one row (H=2048, V=128256, k=10) -- the
cost the paper's trimming attacks (Section 2.3: 2*d*V FLOPs = bytes of bf16 W per token).
The other workloads (row counts 4 and 8, the V_draft sweep 4096..128256 at H=4096, the
1024-row tree-drafting batch and the 512-row full-vocabulary batch) are reported in "sweep".

Timing is "cold": calls rotate over enough distinct copies of W_sub that the footprint
exceeds 1 GiB, so the 256 MB last-level cache cannot serve repeats.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix cores


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-sweep", action="store_true", help="only the headline workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--only", type=str, default=None, help="run a single named workload as the headline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device copy a few times and exit (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE profiler counters)")
    ap.add_argument("--select", action="store_true",
                    help="measure only the vocabulary-size selection call and exit")
    ap.add_argument("--shape", type=str, default=None,
                    help="rows,H,V_draft,k: run this shape as the headline instead (exploration)")
    return ap.parse_args()


def workloads():
    from paper_2603_05210_amd.synth import FULL_VOCAB as V
    w = []
    w.append(dict(name="cfg1_B1", H=2048, rows=1, Vd=V, k=10, peaked=0.0))
    w.append(dict(name="cfg0", H=2048, rows=1, Vd=4096, k=1, peaked=0.0))
    w.append(dict(name="cfg1_B4", H=2048, rows=4, Vd=V, k=10, peaked=0.0))
    w.append(dict(name="cfg1_B8", H=2048, rows=8, Vd=V, k=10, peaked=0.0))
    for vd in (4096, 8192, 16384, 32768, 65536, V):
        w.append(dict(name="cfg2_Vd%d" % vd, H=4096, rows=1, Vd=vd, k=10, peaked=0.0))
    w.append(dict(name="cfg3", H=4096, rows=1024, Vd=32000, k=8, peaked=0.0))
    w.append(dict(name="cfg4", H=4096, rows=512, Vd=V, k=16, peaked=0.05))
    return w


def algorithmic(w):
    """Algorithmic bytes and FLOPs of one step's projection kernel."""
    H, R, Vd, k = w["H"], w["rows"], w["Vd"], w["k"]
    nbytes = 2 * H * Vd + 2 * R * H + 4 * k * R + 8 * k * R
    flops = 2 * R * H * Vd
    return nbytes, flops


class Runner:
    def __init__(self, torch, vt, synth, dev):
        self.torch, self.vt, self.synth, self.dev = torch, vt, synth, dev
        self.W_host = {}
        self.W_dev = {}

    def full_W(self, H):
        import numpy as np
        if H not in self.W_dev:
            Wh = self.synth.gen_W(0, self.synth.FULL_VOCAB, H)
            self.W_host[H] = Wh
            self.W_dev[H] = self.torch.from_numpy(Wh.view(np.int16)).to(self.dev).view(self.torch.bfloat16)
        return self.W_host[H], self.W_dev[H]

    def prepare(self, w):
        import numpy as np
        torch, vt, synth = self.torch, self.vt, self.synth
        Wh, Wd = self.full_W(w["H"])
        ids = synth.zipf_subset(0, synth.FULL_VOCAB, w["Vd"])
        ids_dev = torch.from_numpy(ids).to(self.dev)
        h = synth.gen_h(0, w["rows"], w["H"], peaked_frac=w["peaked"])
        h_dev = torch.from_numpy(h.view(np.int16)).to(self.dev).view(torch.bfloat16)
        # one-time set-up, timed on its own
        W_sub, d2t = vt.vt_build_subset(Wd, ids_dev)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        vt.vt_build_subset(Wd, ids_dev, W_sub, d2t)
        e1.record()
        torch.cuda.synchronize()
        build_ms = e0.elapsed_time(e1)
        nbytes = W_sub.numel() * 2
        n_copies = max(2, -(-(1 << 30) // nbytes))
        copies = [W_sub] + [W_sub.clone() for _ in range(n_copies - 1)]
        ws = torch.empty(max(16, vt.vt_draft_head_workspace_bytes(w["rows"], w["H"], w["Vd"], w["k"])),
                         dtype=torch.uint8, device=self.dev)
        out_ids = torch.empty((w["rows"], w["k"]), dtype=torch.int32, device=self.dev)
        out_lp = torch.empty((w["rows"], w["k"]), dtype=torch.float32, device=self.dev)
        return dict(ids=ids, h=h, h_dev=h_dev, d2t=d2t, copies=copies, ws=ws, out_ids=out_ids, out_lp=out_lp,
                    build_ms=build_ms, n_copies=n_copies)

    def time_steps(self, w, st, steps, warmup):
        torch, vt = self.torch, self.vt
        copies, n = st["copies"], len(st["copies"])

        def step(i):
            vt.vt_draft_head(st["h_dev"], copies[i % n], st["d2t"], w["k"], st["out_ids"], st["out_lp"], st["ws"])

        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(steps):
            step(warmup + i)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        dev_ms = e0.elapsed_time(e1)
        # second pass: HIP events around the projection kernel alone, on the same stream
        vt.vt_kernel_timing_enable(True)
        for i in range(steps):
            step(warmup + i)
        torch.cuda.synchronize()
        n_l, k_ms = vt.vt_kernel_timing_read()
        vt.vt_kernel_timing_enable(False)
        return dict(ms_per_step=max(wall_ms, dev_ms) / steps, dev_ms_per_step=dev_ms / steps,
                    kernel_ms=k_ms / max(n_l, 1), kernel_launches=n_l)


def report(w, st, t):
    nbytes, flops = algorithmic(w)
    regime = "hbm" if w["rows"] <= 16 else "mfma"
    k_s = t["kernel_ms"] * 1e-3
    gbs = nbytes / k_s / 1e9
    tfl = flops / k_s / 1e12
    if regime == "hbm":
        roof = dict(bound="hbm", achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS, traffic=None)
    else:
        roof = dict(bound="mfma", achieved=tfl, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=tfl / MFMA_BF16_PEAK_TFLOPS, traffic=None)
    roof["kernel"] = "gemv_head_kernel" if regime == "hbm" else "gemm_head_kernel"
    roof["kernel_us"] = t["kernel_ms"] * 1e3
    roof["algorithmic_bytes"] = nbytes
    roof["algorithmic_flops"] = flops
    return dict(workload=w["name"], rows=w["rows"], H=w["H"], V_draft=w["Vd"], k=w["k"],
                us_per_step=t["ms_per_step"] * 1e3, device_us_per_step=t["dev_ms_per_step"] * 1e3,
                step_GBps=nbytes / (t["ms_per_step"] * 1e-3) / 1e9, step_TFLOPs=flops / (t["ms_per_step"] * 1e-3) / 1e12,
                build_subset_us=st["build_ms"] * 1e3, w_sub_copies=st["n_copies"], roofline=roof)


def cpu_baseline(runner, w, st):
    """The CPU oracle, as it stands, on the headline workload (bounded to ~10-30 s)."""
    from oracle import vt_oracle as vo
    Wh, _ = runner.full_W(w["H"])
    ids = st["ids"]
    W_sub = Wh if len(ids) == Wh.shape[0] else Wh[ids]
    rows = st["h"].shape[0]
    # bounded sample: at most 8 rows of the batch, repeated until ~10 s have passed
    r_use = min(rows, 8)
    h = st["h"][:r_use]
    reps, t_total = 0, 0.0
    while t_total < 10.0 and reps < 5000:
        t0 = time.perf_counter()
        vo.draft_head(h, W_sub, ids, w["k"], want_logits=False)
        t_total += time.perf_counter() - t0
        reps += 1
    per_row_us = t_total / reps / r_use * 1e6
    return dict(value=per_row_us * rows, unit="us/step", cores=vo.num_threads(), kind="oracle",
                sample="%d of %d rows x full V_draft=%d, %d repetitions, %.1f s of CPU time; scaled by rows"
                       % (r_use, rows, len(ids), reps, t_total))


def kernel_source_hash():
    """sha256 over the HIP sources of the draft-head kernels (everything but the selection and
    coverage files): recorded with profiler counters so stale counters are not reported."""
    import hashlib
    h = hashlib.sha256()
    for f in sorted((ROOT / "paper_2603_05210_amd" / "csrc").glob("*")):
        if f.suffix in (".hip", ".h") and not f.name.startswith(("vt_select", "vt_coverage")):
            h.update(f.name.encode())
            h.update(f.read_bytes())
    return h.hexdigest()


def recorded_traffic(workload_name):
    """HBM bytes per launch of the dominant kernel from profiles/hbm_traffic.json (rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE, scaled by the same counters' reading for a plain copy), or None when
    the kernels changed since the counters were taken."""
    f = ROOT / "profiles" / "hbm_traffic.json"
    if not f.exists():
        return None
    rec = json.loads(f.read_text())
    if rec.get("source_sha256") != kernel_source_hash():
        return None
    w = rec.get("workloads", {}).get(workload_name)
    return None if w is None else w.get("traffic_bytes")


def calibrate_copy():
    import torch
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy_bytes": n, "reads": n, "writes": n, "launches": 5}))


def selector_bench(torch, vt, synth, dev, with_cpu, n_tokens=32 * 1024 * 1024, calls=5):
    """The vocabulary-size selection (Eq. 1-5) on a Zipf(1.1) stream over LLaMA-3's vocabulary
    with Table 1's constants: whole-call time (kernels + the call's one synchronisation)."""
    V, d = synth.FULL_VOCAB, 4096
    F_fixed = (100.7 + 436.2 + 50.3) * 1e6
    alpha, c_min, k_min = 0.5, 0.9, 1024
    tokens = synth.zipf_token_stream(0, V, n_tokens)
    t_dev = torch.from_numpy(tokens).to(dev)
    ws = torch.empty(vt.vt_select_vocab_workspace_bytes(V), dtype=torch.uint8, device=dev)
    res = None
    for _ in range(2):
        res, _, _, _ = vt.vt_select_vocab(t_dev, V, d, F_fixed, alpha, c_min, k_min, V, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(calls):
        res, _, _, _ = vt.vt_select_vocab(t_dev, V, d, F_fixed, alpha, c_min, k_min, V, workspace=ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / calls
    out = dict(workload="select_vocab: V=%d d=%d n_tokens=%d Zipf(1.1) alpha=%g c_min=%g" % (V, d, n_tokens, alpha, c_min),
               ms_per_call=ms, Mtokens_per_s=n_tokens / ms / 1e3, stream_GBps=4.0 * n_tokens / (ms * 1e-3) / 1e9,
               k_star=int(res.k_star), C=res.C, R=res.R, U=res.U)
    # coverage of the selected vocabulary on the same stream (Table 4's two ratios)
    _, _, _, ids = vt.vt_select_vocab(t_dev, V, d, F_fixed, alpha, c_min, k_min, V, workspace=ws)
    t2d = vt.vt_build_t2d(ids.contiguous(), V)
    cws = torch.empty(vt.vt_coverage_workspace_bytes(V), dtype=torch.uint8, device=dev)
    cov, _ = vt.vt_coverage(t_dev, t2d, workspace=cws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(calls):
        cov, _ = vt.vt_coverage(t_dev, t2d, workspace=cws)
    torch.cuda.synchronize()
    cms = (time.perf_counter() - t0) * 1e3 / calls
    out["coverage"] = dict(ms_per_call=cms, Mtokens_per_s=n_tokens / cms / 1e3,
                           stream_GBps=4.0 * n_tokens / (cms * 1e-3) / 1e9, freq_coverage=cov.freq_coverage,
                           unique_coverage=cov.unique_coverage)
    if with_cpu:
        from oracle import vs_oracle as vs
        sample = tokens[: 8 * 1024 * 1024]
        t0 = time.perf_counter()
        ora = vs.select_vocab(sample, V, d, F_fixed, alpha, c_min, k_min, V)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = dict(value=sample.size / dt / 1e6, unit="Mtokens/s", cores=1, kind="oracle",
                                   sample="first %d tokens of the same stream, one call" % sample.size,
                                   k_star=ora.k_star)
    return out


def main():
    args = parse_args()
    if args.calibrate_copy:
        calibrate_copy()
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the head runs on exactly one GPU here (the head shards by vocabulary or by rows "
              "without changing the per-GPU kernel); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2603_05210_amd as vt
    from paper_2603_05210_amd import synth

    if not vt.LIB_PATH.exists():
        from paper_2603_05210_amd import build as vt_build
        vt_build.build()
    vt.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.select:
        print(json.dumps({"selector": selector_bench(torch, vt, synth, dev, with_cpu=not args.no_cpu)}))
        return
    runner = Runner(torch, vt, synth, dev)

    wl = workloads()
    if args.shape:
        r_, h_, v_, k_ = (int(x) for x in args.shape.split(","))
        wl = [dict(name="shape_%s" % args.shape.replace(",", "x"), H=h_, rows=r_, Vd=v_, k=k_, peaked=0.0)]
        args.only = wl[0]["name"]
    if args.only:
        wl = [w for w in wl if w["name"] == args.only]
        assert wl, "unknown workload"
    head = wl[0]
    st = runner.prepare(head)
    torch.cuda.synchronize()
    t = runner.time_steps(head, st, args.steps, args.warmup)
    torch.cuda.synchronize()
    head_rep = report(head, st, t)
    head_rep["roofline"]["traffic"] = recorded_traffic(head["name"])
    cpu = None if args.no_cpu else cpu_baseline(runner, head, st)
    del st
    sweep = []
    if not args.no_sweep and not args.only:
        for w in wl[1:]:
            s = runner.prepare(w)
            steps = max(20, min(args.steps, 100))
            sweep.append(report(w, s, runner.time_steps(w, s, steps, min(args.warmup, 10))))
            del s
            torch.cuda.empty_cache()

    selector = None
    if not args.no_sweep and not args.only:
        selector = selector_bench(torch, vt, synth, dev, with_cpu=not args.no_cpu)

    out = {
        "metric": "draft_lm_head_us_per_step",
        "value": head_rep["us_per_step"],
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head_rep["us_per_step"] / 1e3,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic (seeded N(0,0.02) W, N(0,1) h, Zipf(1.1)-ranked subsets); cold: rotating W_sub copies > 1 GiB",
        "config": {"workload": "%s: rows=%d H=%d V_draft=%d k=%d (untrimmed baseline head, identity d2t)"
                               % (head["name"], head["rows"], head["H"], head["Vd"], head["k"]),
                   "device_us_per_step": head_rep["device_us_per_step"],
                   "build_subset_us": head_rep["build_subset_us"]},
        "roofline": head_rep["roofline"],
        "cpu_baseline": cpu,
        "sweep": sweep,
        "selector": selector,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
