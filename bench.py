#!/usr/bin/env python3
"""Benchmark of the trimmed-vocabulary draft LM head on one MI355X.

A "step" is one draft step through the C ABI: vt_draft_head (projection over the draft
vocabulary with fused softmax statistics and top-k, merge, d2t remap) on inputs already in
HBM.  vt_build_subset is the one-time set-up per draft vocabulary (Section 2.1 of the paper)
and is timed separately ("build_subset_us"), not as part of a step.

Headline workload: the metric's own curve -- one row, H = 4096 (the paper's d), V_draft swept
from 4096 to the full 128 256 (Section 2.3: the head costs 2*d*k FLOPs = bytes of bf16 W_sub
per token); `value` is the full-vocabulary end of the curve, every other point, the three
vocabulary sizes the paper itself selects (Sections 2.6 and 3.2), the 2048-wide heads and the
two tree-drafting batches are in "sweep".

Protocol per workload, both flagged in the output:
  cold   calls rotate over enough distinct copies of W_sub that the footprint exceeds 1 GiB,
         so the 256 MB last-level cache cannot serve repeats (roofline fractions use this);
  warm   the same W_sub every call (what a serving loop sees at small V_draft: a cache number).
Each mode: `steps` back-to-back calls between one event pair (dense-loop mean, the figure the
roofline fraction is computed from) and `steps` calls each between its own event pair (p10 /
median / p90; these carry about 2 us of event overhead per call).  All events are recorded on
the stream the kernels are launched on.  Prints ONE JSON line.
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
HEADLINE = "cfg2_Vd128256"
PAPER_SIZES = (4380, 6521, 13264)   # function calling, NER (Section 3.2), general (Section 2.6)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-sweep", action="store_true", help="only the headline workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline legs")
    ap.add_argument("--no-warm", action="store_true", help="skip the warm (same W_sub every call) mode")
    ap.add_argument("--no-percall", action="store_true", help="skip the per-call event pass (dense loop only)")
    ap.add_argument("--only", type=str, default=None, help="run a single named workload as the headline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device copy a few times and exit (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE profiler counters)")
    ap.add_argument("--calibrate-gemm", action="store_true",
                    help="time the vendor library's plain bf16 GEMM (torch.matmul: no softmax, no top-k, bf16 logits "
                         "stored) on the two tree-drafting shapes, with the benchmark's operands and with constant "
                         "ones: what a GEMM alone reaches on this GPU at these sizes")
    ap.add_argument("--select", action="store_true",
                    help="measure only the vocabulary-size selection call and exit")
    ap.add_argument("--operands", choices=("gaussian", "zero_h", "const"), default="gaussian",
                    help="operand values of the head workloads (same shapes, same kernels): the seeded Gaussian inputs, "
                         "a zero hidden state, or constant W_sub and h -- how much of the matrix-core regime's time is "
                         "the data toggling the datapath rather than the schedule")
    ap.add_argument("--shape", type=str, default=None,
                    help="rows,H,V_draft,k: run this shape as the headline instead (exploration)")
    return ap.parse_args()


def workloads():
    """The headline first, then the rest of its curve, then the other configurations."""
    from paper_2603_05210_amd.synth import FULL_VOCAB as V
    w = [dict(name=HEADLINE, H=4096, rows=1, Vd=V, k=10, peaked=0.0)]
    for vd in (4096, 8192, 16384, 32768, 65536):
        w.append(dict(name="cfg2_Vd%d" % vd, H=4096, rows=1, Vd=vd, k=10, peaked=0.0))
    for vd in PAPER_SIZES:
        w.append(dict(name="paper_Vd%d" % vd, H=4096, rows=1, Vd=vd, k=10, peaked=0.0))
    w.append(dict(name="cfg0", H=2048, rows=1, Vd=4096, k=1, peaked=0.0))
    for b in (1, 4, 8):
        w.append(dict(name="cfg1_B%d" % b, H=2048, rows=b, Vd=V, k=10, peaked=0.0))
    # one tree-drafting step of one sequence (8 nodes) and of four (32 nodes) over the vocabulary Section 2.6 selects
    w.append(dict(name="tree_rows8_Vd13264", H=4096, rows=8, Vd=13264, k=8, peaked=0.0))
    w.append(dict(name="tree_rows32_Vd13264", H=4096, rows=32, Vd=13264, k=8, peaked=0.0))
    w.append(dict(name="cfg3", H=4096, rows=1024, Vd=32000, k=8, peaked=0.0))
    w.append(dict(name="cfg4", H=4096, rows=512, Vd=V, k=16, peaked=0.05))
    # the one-row step over a compressed W_sub, with its neighbours fused in, and the fusion layer ahead of it
    for vd in (13264, V):
        w.append(dict(name="fp8_Vd%d" % vd, kind="head_q", fmt=1, H=4096, rows=1, Vd=vd, k=10, peaked=0.0))
        w.append(dict(name="mxfp4_Vd%d" % vd, kind="head_q", fmt=2, H=4096, rows=1, Vd=vd, k=10, peaked=0.0))
    # a tree-drafting step of 8 nodes over the compressed forms
    w.append(dict(name="fp8_rows8_Vd13264", kind="head_q", fmt=1, H=4096, rows=8, Vd=13264, k=8, peaked=0.0))
    w.append(dict(name="mxfp4_rows8_Vd13264", kind="head_q", fmt=2, H=4096, rows=8, Vd=13264, k=8, peaked=0.0))
    w.append(dict(name="fused_Vd13264", kind="head_fused", H=4096, rows=1, Vd=13264, k=10, peaked=0.0))
    w.append(dict(name="fused_rows8_Vd13264", kind="head_fused", H=4096, rows=8, Vd=13264, k=8, peaked=0.0))
    w.append(dict(name="fusion_B1", kind="fusion", H=4096, rows=1, Vd=4096, k=1, peaked=0.0))
    w.append(dict(name="fusion_B64", kind="fusion", H=4096, rows=64, Vd=4096, k=1, peaked=0.0))
    for x in w:
        x.setdefault("kind", "head")
    return w


def describe(w):
    from paper_2603_05210_amd.synth import FULL_VOCAB as V
    if w.get("kind") == "fusion":
        return "%s: feature-fusion projection rows=%d d_in=%d d_out=%d" % (w["name"], w["rows"], 3 * w["H"], w["H"])
    kind = "untrimmed head, identity d2t" if w["Vd"] == V else "Zipf(1.1)-ranked draft vocabulary of a %d-token head" % V
    return "%s: rows=%d H=%d V_draft=%d k=%d (%s)" % (w["name"], w["rows"], w["H"], w["Vd"], w["k"], kind)


def algorithmic(w):
    """Algorithmic bytes and FLOPs of one step's projection kernel."""
    H, R, Vd, k = w["H"], w["rows"], w["Vd"], w["k"]
    kind = w.get("kind", "head")
    if kind == "fusion":           # g = x . W_fc^T with d_in = 3H, d_out = H (Section 2.3: 2*3d*d FLOPs per row)
        return 2 * 3 * H * H + 2 * R * 3 * H + 2 * R * H, 2 * R * 3 * H * H
    wbytes = 2 * H * Vd
    if kind == "head_q":           # codes + scales
        wbytes = H * Vd + 4 * Vd if w["fmt"] == 1 else H * Vd // 2 + (H // 32) * Vd
    extra = 2 * H + 4 * R if kind == "head_fused" else 0     # gamma, parent scores
    nbytes = wbytes + 2 * R * H + 4 * k * R + 8 * k * R + extra
    flops = 2 * R * H * Vd
    return nbytes, flops


def percentile(sorted_vals, q):
    if not sorted_vals:
        return None
    i = min(len(sorted_vals) - 1, max(0, int(round(q * (len(sorted_vals) - 1)))))
    return sorted_vals[i]


class Runner:
    def __init__(self, torch, vt, synth, dev):
        self.torch, self.vt, self.synth, self.dev = torch, vt, synth, dev
        self.W_host = {}
        self.W_dev = {}
        self.operands = "gaussian"

    def full_W(self, H):
        import numpy as np
        if H not in self.W_dev:
            Wh = self.synth.gen_W(0, self.synth.FULL_VOCAB, H)
            self.W_host[H] = Wh
            self.W_dev[H] = self.torch.from_numpy(Wh.view(np.int16)).to(self.dev).view(self.torch.bfloat16)
        return self.W_host[H], self.W_dev[H]

    def drop_W(self, H):
        self.W_host.pop(H, None)
        self.W_dev.pop(H, None)

    def prepare_fusion(self, w):
        import numpy as np
        torch, vt, synth = self.torch, self.vt, self.synth
        d = w["H"]
        x = synth.gen_h(0, w["rows"], 3 * d)
        Wfc = synth.gen_W(7, d, 3 * d)
        to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(self.dev).view(torch.bfloat16)
        Wfc_dev = to_dev(Wfc)
        n_copies = max(2, -(-(1 << 30) // (Wfc.size * 2)))
        return dict(kind="fusion", x=x, Wfc=Wfc, x_dev=to_dev(x), copies=[Wfc_dev] + [Wfc_dev.clone() for _ in range(n_copies - 1)],
                    g=torch.empty((w["rows"], d), dtype=torch.bfloat16, device=self.dev), build_ms=0.0, n_copies=n_copies)

    def prepare(self, w):
        import numpy as np
        torch, vt, synth = self.torch, self.vt, self.synth
        kind = w.get("kind", "head")
        if kind == "fusion":
            return self.prepare_fusion(w)
        Wh, Wd = self.full_W(w["H"])
        ids = synth.zipf_subset(0, synth.FULL_VOCAB, w["Vd"])
        ids_dev = torch.from_numpy(ids).to(self.dev)
        h = synth.gen_h(0, w["rows"], w["H"], peaked_frac=w["peaked"])
        h_dev = torch.from_numpy(h.view(np.int16)).to(self.dev).view(torch.bfloat16)
        # one-time set-up, timed on its own
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if kind == "head_q":
            vt.vt_build_subset_q(Wd, ids_dev, w["fmt"])
            torch.cuda.synchronize()
            e0.record()
            codes, scales, d2t = vt.vt_build_subset_q(Wd, ids_dev, w["fmt"])
            e1.record()
            first = (codes, scales)
            nbytes = codes.numel() + scales.numel() * scales.element_size()
        else:
            W_sub, d2t = vt.vt_build_subset(Wd, ids_dev)
            torch.cuda.synchronize()
            e0.record()
            vt.vt_build_subset(Wd, ids_dev, W_sub, d2t)
            e1.record()
            first = (W_sub,)
            nbytes = W_sub.numel() * 2
        torch.cuda.synchronize()
        build_ms = e0.elapsed_time(e1)
        n_copies = max(2, -(-(1 << 30) // nbytes))
        copies = [first] + [tuple(t.clone() for t in first) for _ in range(n_copies - 1)]
        if kind == "head_q":
            need = vt.vt_draft_head_q_workspace_bytes(w["fmt"], w["rows"], w["H"], w["Vd"], w["k"])
        else:   # the fused call's need covers the plain call's
            need = vt.vt_draft_head_fused_workspace_bytes(w["rows"], w["H"], w["Vd"], w["k"])
        ws = vt.new_workspace(need, self.dev)
        out_ids = torch.empty((w["rows"], w["k"]), dtype=torch.int32, device=self.dev)
        out_lp = torch.empty((w["rows"], w["k"]), dtype=torch.float32, device=self.dev)
        if self.operands == "zero_h":
            h_dev.zero_()
        elif self.operands == "const":
            h_dev.fill_(1.0)
            for c in copies:
                c[0].fill_(0.0201 if kind != "head_q" else 57)
        st = dict(kind=kind, ids=ids, h=h, h_dev=h_dev, d2t=d2t, copies=copies, ws=ws, out_ids=out_ids, out_lp=out_lp,
                  build_ms=build_ms, n_copies=n_copies)
        if kind == "head_fused":
            gamma = synth.f32_to_bf16((1.0 + 0.1 * synth.normal(0, 9, 0, w["H"])).astype(np.float32))
            parent = (-np.abs(synth.normal(0, 10, 0, w["rows"]))).astype(np.float32)
            st.update(gamma=gamma, parent=parent, gamma_dev=torch.from_numpy(gamma.view(np.int16)).to(self.dev).view(torch.bfloat16),
                      parent_dev=torch.from_numpy(parent).to(self.dev))
        return st

    def time_mode(self, w, st, steps, warmup, cold, percall):
        """Dense-loop mean and per-call percentiles of one mode (cold: rotating W_sub copies)."""
        torch, vt = self.torch, self.vt
        copies = st["copies"] if cold else st["copies"][:1]
        n = len(copies)

        kind = st["kind"]
        if kind == "fusion":
            def step(i):
                vt.vt_feature_fusion(st["x_dev"], copies[i % n], st["g"])
        elif kind == "head_q":
            def step(i):
                c = copies[i % n]
                vt.vt_draft_head_q(st["h_dev"], c[0], c[1], w["fmt"], st["d2t"], w["k"], st["out_ids"], st["out_lp"], st["ws"])
        elif kind == "head_fused":
            def step(i):
                vt.vt_draft_head_fused(st["h_dev"], st["gamma_dev"], 1e-5, copies[i % n][0], st["d2t"], w["k"], st["parent_dev"],
                                       st["out_ids"], st["out_lp"], st["ws"])
        else:
            def step(i):
                vt.vt_draft_head(st["h_dev"], copies[i % n][0], st["d2t"], w["k"], st["out_ids"], st["out_lp"], st["ws"])

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
        wall_us = (time.perf_counter() - t0) * 1e6 / steps
        dense_us = e0.elapsed_time(e1) * 1e3 / steps
        out = dict(mode="cold" if cold else "warm", dense_loop_us=dense_us, wall_us=wall_us,
                   us_per_step=max(dense_us, wall_us))
        if percall:
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for i, (a, b) in enumerate(evs):
                a.record()
                step(warmup + i)
                b.record()
            torch.cuda.synchronize()
            v = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
            out.update(percall_p10_us=percentile(v, 0.10), percall_median_us=percentile(v, 0.50),
                       percall_p90_us=percentile(v, 0.90), percall_calls=steps)
        return out


def report(w, st, cold, warm):
    nbytes, flops = algorithmic(w)
    # up to 64 rows the step is bound by reading W_sub once (at most 64 FLOP per byte); so is the fusion layer at 64 rows
    regime = "hbm" if (w["rows"] <= 64 or w.get("kind") == "fusion") else "mfma"
    t_s = cold["us_per_step"] * 1e-6   # dense-loop device time per step (wall clock if that is larger)
    gbs = nbytes / t_s / 1e9
    tfl = flops / t_s / 1e12
    if regime == "hbm":
        roof = dict(bound="hbm", achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS, traffic=None)
    else:
        roof = dict(bound="mfma", achieved=tfl, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=tfl / MFMA_BF16_PEAK_TFLOPS, traffic=None)
    kind = w.get("kind", "head")
    roof["kernel"] = ("feature-fusion kernel (whole call)" if kind == "fusion" else "streaming head kernel (whole step)" if regime == "hbm"
                      else "gemm_head_kernel + merge_kernel (whole step)")
    roof["from"] = "cold dense-loop time per step"
    roof["algorithmic_bytes"] = nbytes
    roof["algorithmic_flops"] = flops
    roof["traffic"] = recorded_traffic(w["name"])
    rep = dict(workload=w["name"], rows=w["rows"], H=w["H"], V_draft=w["Vd"], k=w["k"],
               us_per_step=cold["us_per_step"], cold=cold, warm=warm,
               build_subset_us=st["build_ms"] * 1e3, w_sub_copies=st["n_copies"], roofline=roof)
    if warm is not None:
        rep["warm_effective_GBps"] = nbytes / (warm["us_per_step"] * 1e-6) / 1e9   # may exceed HBM peak: served by the last-level cache
    return rep


def cpu_baseline(runner, w, st, budget_s):
    """The CPU oracle, as it stands, on a bounded sample of the workload's rows."""
    from oracle import vt_oracle as vo
    kind = st["kind"]
    if kind == "fusion":
        from oracle import vp_oracle as vp
        rows = st["x"].shape[0]
        r_use = min(rows, 4)
        reps, t_total = 0, 0.0
        while t_total < budget_s and reps < 5000:
            t0 = time.perf_counter()
            vp.feature_fusion(st["x"][:r_use], st["Wfc"])
            t_total += time.perf_counter() - t0
            reps += 1
        return dict(value=t_total / reps / r_use * 1e6 * rows, unit="us/step", cores=vo.num_threads(), kind="oracle",
                    sample="%d of %d rows, %d repetitions, %.1f s of CPU time; scaled by rows" % (r_use, rows, reps, t_total))
    Wh, _ = runner.full_W(w["H"])
    ids = st["ids"]
    W_sub = Wh if len(ids) == Wh.shape[0] else Wh[ids]
    rows = st["h"].shape[0]
    r_use = min(rows, 4)
    h = st["h"][:r_use]
    reps, t_total = 0, 0.0
    if kind == "head_q":
        from oracle import vq_oracle as vq
        codes, scales = vq.quantize(W_sub, w["fmt"])        # set-up, not timed
        call = lambda: vq.draft_head_q(h, codes, scales, w["fmt"], ids, w["k"], want_logits=False)
    elif kind == "head_fused":
        from oracle import vp_oracle as vp
        call = lambda: vp.head_fused(h, st["gamma"], 1e-5, W_sub, ids, w["k"], st["parent"][:r_use])
    else:
        call = lambda: vo.draft_head(h, W_sub, ids, w["k"], want_logits=False)
    while t_total < budget_s and reps < 5000:
        t0 = time.perf_counter()
        call()
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
        if f.suffix in (".hip", ".h", ".cpp") and not f.name.startswith(("vt_select", "vt_coverage")):
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


def calibrate_gemm(steps=50):
    """Dense loop of torch.matmul(h, W_sub^T) on the cfg3 / cfg4 shapes (and a large square one)."""
    import torch
    from paper_2603_05210_amd import synth
    dev = "cuda:0"
    out = []
    for name, rows, H, Vd in (("cfg3", 1024, 4096, 32000), ("cfg4", 512, 4096, synth.FULL_VOCAB), ("square_8192", 8192, 8192, 8192)):
        for fill in ("gaussian", "const"):
            if fill == "gaussian":
                g = torch.Generator(device=dev).manual_seed(0)
                h = torch.randn(rows, H, device=dev, generator=g).to(torch.bfloat16)
                W = (torch.randn(Vd, H, device=dev, generator=g) * 0.02).to(torch.bfloat16)
            else:
                h = torch.full((rows, H), 1.0, device=dev, dtype=torch.bfloat16)
                W = torch.full((Vd, H), 0.02, device=dev, dtype=torch.bfloat16)
            z = torch.empty(rows, Vd, device=dev, dtype=torch.bfloat16)
            for _ in range(10):
                torch.matmul(h, W.t(), out=z)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                torch.matmul(h, W.t(), out=z)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / steps
            fl = 2.0 * rows * H * Vd
            out.append({"shape": name, "rows": rows, "H": H, "V_draft": Vd, "operands": fill, "us_per_call": round(us, 1),
                        "tflops": round(fl / us / 1e6, 1), "frac_of_2500": round(fl / us / 1e6 / 2500.0, 3)})
            del h, W, z
            torch.cuda.empty_cache()
    print(json.dumps({"calibrate_gemm": out, "steps": steps, "library": "torch.matmul (hipBLASLt / rocBLAS)"}))


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
    # both calls are bound by reading the 4-byte token stream once: achieved = stream bytes over the whole
    # call (for the selection that includes ranking 128 Ki frequencies and the call's synchronisation)
    out["roofline"] = dict(bound="hbm", achieved=out["stream_GBps"], peak=HBM_PEAK_GBS, unit="GB/s",
                           frac=out["stream_GBps"] / HBM_PEAK_GBS, traffic=None)
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
    out["coverage"]["roofline"] = dict(bound="hbm", achieved=out["coverage"]["stream_GBps"], peak=HBM_PEAK_GBS, unit="GB/s",
                                       frac=out["coverage"]["stream_GBps"] / HBM_PEAK_GBS, traffic=None)
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
    if args.calibrate_gemm:
        calibrate_gemm()
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
    runner.operands = args.operands

    wl = workloads()
    if args.shape:
        r_, h_, v_, k_ = (int(x) for x in args.shape.split(","))
        wl = [dict(name="shape_%s" % args.shape.replace(",", "x"), H=h_, rows=r_, Vd=v_, k=k_, peaked=0.0)]
        args.only = wl[0]["name"]
    if args.only:
        wl = [w for w in wl if w["name"] == args.only]
        assert wl, "unknown workload"
    if args.no_sweep:
        wl = wl[:1]
    # group by hidden size so that only one full matrix is resident at a time
    order = [wl[0]] + sorted(wl[1:], key=lambda w: (w["H"] != wl[0]["H"], w["H"]))

    reports, cpus = {}, {}
    for n, w in enumerate(order):
        if n > 0 and w["H"] != order[n - 1]["H"]:
            runner.drop_W(order[n - 1]["H"])
            torch.cuda.empty_cache()
        st = runner.prepare(w)
        torch.cuda.synchronize()
        steps, warmup = (args.steps, args.warmup) if n == 0 else (max(20, args.steps), max(5, args.warmup))
        cold = runner.time_mode(w, st, steps, warmup, True, not args.no_percall)
        warm = None if args.no_warm else runner.time_mode(w, st, steps, warmup, False, not args.no_percall)
        reports[w["name"]] = report(w, st, cold, warm)
        if not args.no_cpu:
            cpus[w["name"]] = cpu_baseline(runner, w, st, 8.0 if n == 0 else 1.0)
            reports[w["name"]]["cpu_baseline"] = cpus[w["name"]]
        del st
        torch.cuda.empty_cache()

    head = wl[0]
    head_rep = reports[head["name"]]
    sweep = [reports[w["name"]] for w in wl[1:]]
    selector = None
    if not args.no_sweep and not args.only:
        runner.drop_W(order[-1]["H"])
        torch.cuda.empty_cache()
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
        "data": "synthetic (seeded N(0,0.02) W, N(0,1) h, Zipf(1.1)-ranked subsets); value = cold: rotating W_sub copies > 1 GiB"
                + ("" if args.operands == "gaussian" else "; OPERAND ABLATION: %s" % args.operands),
        "config": {"workload": describe(head), "mode": "cold",
                   "percall_median_us": head_rep["cold"].get("percall_median_us"),
                   "percall_p10_us": head_rep["cold"].get("percall_p10_us"),
                   "percall_p90_us": head_rep["cold"].get("percall_p90_us"),
                   "warm_us_per_step": None if head_rep["warm"] is None else head_rep["warm"]["us_per_step"],
                   "build_subset_us": head_rep["build_subset_us"]},
        "roofline": head_rep["roofline"],
        "cpu_baseline": cpus.get(head["name"]),
        "sweep": sweep,
        "selector": selector,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
