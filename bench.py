#!/usr/bin/env python3
"""Benchmark of the adapted quantized linear layer hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch of a LLaMA-shaped layer stack: for every
projection of the workload, in sequence on one shared workspace,
    block-wise quantize -> adapted forward (s*U kept) -> backward (dX, dA, dB),
then the tile product H = A B and the requantizing INT4 merge of ALL projections back to back (the batch the
merge is meant to be timed on).  Default workload: the LLaMA-65B-shaped layer (seven projections, T = 8192,
double-quantized block scales, rank 128), the largest single-GPU configuration.  All inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

value        algorithmic fwd+bwd flops of all projections (4*T*d_in*d_out + 6*T*r*(d_in+d_out) each) over the
             wall time of the whole step, TFLOP/s.
roofline     the forward dequantize-and-contract kernel on the workload's largest projection, timed with HIP
             events that the library records on the launch stream around that one launch, against the dense
             bf16 MFMA peak; frac is computed from that shape's own flops.
kernels      the other kernels of the same projection (backward GEMM, narrow adapter GEMMs, token contractions,
             quantize) from an untimed pass with one event pair per kernel, and the seven-matrix merge batch.
configs      the same measurement on the other workloads (7B attention projection, 7B MLP, 13B stack with its
             rank sweep), fewer steps each.
cpu_baseline the fp64 CPU oracle on a bounded sample (a few token rows of each distinct projection shape),
             extrapolated linearly in tokens and projection count, labelled as such.
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs, as recorded by the profile step in
    profiles/hbm_traffic.txt (lines `workload kernel bytes`); None when that pair has not been profiled."""
    try:
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) >= 3 and not line.startswith("#") and f[0] == workload and f[1] == kernel:
                return int(float(f[2]))
    except OSError:
        pass
    return None


VALU_FILE = os.path.join(ROOT, "profiles", "valu_counters.txt")


def measured_valu(workload: str, kernel: str):
    """Vector-ALU figures of a streaming kernel from the rocprofv3 SQ counter runs, as recorded by the profile step
    in profiles/valu_counters.txt (lines `workload kernel lane-instructions-per-weight-element busy-share`): a kernel
    whose vector ALU is busy most of the time is bound by that, not by the HBM rate it is priced against."""
    try:
        for line in open(VALU_FILE):
            f = line.split()
            if len(f) >= 4 and not line.startswith("#") and f[0] == workload and f[1] == kernel:
                return {"valu_lane_insts_per_element": float(f[2]), "valu_busy": float(f[3])}
    except OSError:
        pass
    return None


class Stack:
    """Device state of one workload: per-projection weights, adapters, outputs; shared activations and scratch."""

    def __init__(self, wl, rank, dev):
        import numpy as np
        import torch
        from paper_2407_17029_amd import binding as qb
        from paper_2407_17029_amd import synth
        self.wl, self.lam, self.dev, self.qb = wl, wl.lam, dev, qb
        self.T = T = wl.tokens
        self.cb = synth.codebook_nf4_style()
        self.scale_mode = qb.SCALES_E4M3_GROUPED if wl.scale_mode else qb.SCALES_FP32
        widths_in = sorted({p.d_in for p in wl.projections})
        widths_out = sorted({p.d_out for p in wl.projections})

        # seeded host tensors, drawn concurrently (the generators release the interpreter lock); the streams
        # and distributions are those of synth.make_layer, one seed per projection / activation width
        def job_w(i, p):
            return ("W", i), synth.base_weight(wl.seed + 1 + i, 0, p.d_out, p.d_in)

        def job_x(d):
            return ("X", d), synth.f32_to_bf16_bits(synth.normal_f32(wl.seed + 50, d, (T, d)))

        def job_dy(d):
            return ("dY", d), synth.f32_to_bf16_bits(synth.normal_f32(wl.seed + 60, d, (T, d)))

        jobs = [(job_w, (i, p)) for i, p in enumerate(wl.projections)]
        jobs += [(job_x, (d,)) for d in widths_in] + [(job_dy, (d,)) for d in widths_out]
        with cf.ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
            host = dict(f.result() for f in [pool.submit(fn, *a) for fn, a in jobs])
        self.host = host
        self.X = {d: self._bf16_dev(host[("X", d)]) for d in widths_in}
        self.dY = {d: self._bf16_dev(host[("dY", d)]) for d in widths_out}
        self.Y = {d: torch.empty((T, d), dtype=torch.bfloat16, device=dev) for d in widths_out}
        self.dX = {d: torch.empty((T, d), dtype=torch.bfloat16, device=dev) for d in widths_in}
        self.proj = []
        for i, p in enumerate(wl.projections):
            W = torch.from_numpy(host[("W", i)]).to(dev)
            # the tile-ordered second copy of the codes serves the dequantize-in-kernel contraction of short
            # batches; at this token count the calls dequantize the row-major codes once, so none is asked for
            qw = qb.qblora_quantize_blockwise(W, wl.block, qb.QUANT_ABSMAX_CODEBOOK, self.cb, self.scale_mode,
                                              tiled=T < qb.qblora_dense_min_tokens())
            self.proj.append(dict(p=p, W=W, qw=qw, merged=None,
                                  H=torch.empty((p.d_in // wl.lam, p.d_out // wl.lam), dtype=torch.float32, device=dev)))
        self.set_rank(rank)

    def _bf16_dev(self, bits):
        import numpy as np
        import torch
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(self.dev)

    def set_rank(self, rank):
        """(Re)builds what depends on the adapter rank: A, B, gradient buffers, workspace, saved activation."""
        import numpy as np
        import torch
        from paper_2407_17029_amd import synth
        qb, wl, lam, T, dev = self.qb, self.wl, self.lam, self.T, self.dev
        self.rank, self.R = rank, wl.lam * rank
        R = self.R
        self.ws = self.saved = None
        need = saved = 0
        for i, st in enumerate(self.proj):
            p = st["p"]
            A = synth.uniform_f32(wl.seed + 1 + i + 100 * rank, 3, (p.d_in // lam, R), 1.0 / np.sqrt(p.d_in / lam))
            B = synth.normal_f32(wl.seed + 1 + i + 100 * rank, 4, (R, p.d_out // lam), 0.01)
            self.host[("AB", i)] = (synth.f32_to_bf16_bits(A), synth.f32_to_bf16_bits(B))
            st["ad"] = ad = qb.Adapter(self._bf16_dev(self.host[("AB", i)][0]), self._bf16_dev(self.host[("AB", i)][1]),
                                       lam, lam, wl.s)
            st["dA"] = torch.empty((p.d_in // lam, R), dtype=torch.float32, device=dev)
            st["dB"] = torch.empty((R, p.d_out // lam), dtype=torch.float32, device=dev)
            need = max(need, qb.qblora_linear_fwd_workspace_bytes(st["qw"], ad, T),
                       qb.qblora_linear_bwd_workspace_bytes(st["qw"], ad, T))
            saved = max(saved, qb.qblora_saved_bytes(ad, T))
        self.ws = torch.empty(need + 256, dtype=torch.uint8, device=dev)
        self.saved = torch.empty(saved, dtype=torch.uint8, device=dev)
        for st in self.proj:
            p = st["p"]
            st["merged"] = qb.qablora_merge_quantize(st["qw"], qb.qblora_tile_product(st["ad"], p.d_in, p.d_out, st["H"], self.ws),
                                                     lam, lam, wl.s, qb.MERGE_REQUANT_MINMAX, out=st["merged"])

    def layer_pass(self, st, before_phase=None):
        """quantize -> forward -> backward of one projection; `before_phase(name)` (benchmark hook) runs in front of each."""
        qb, wl, p = self.qb, self.wl, st["p"]
        if before_phase:
            before_phase("quantize")
        qb.qblora_quantize_blockwise(st["W"], wl.block, qb.QUANT_ABSMAX_CODEBOOK, self.cb, self.scale_mode, out=st["qw"])
        if before_phase:
            before_phase("fwd")
        qb.qblora_linear_fwd(st["qw"], st["ad"], self.X[p.d_in], self.Y[p.d_out], self.ws, saved=self.saved)
        if before_phase:
            before_phase("bwd")
        qb.qblora_linear_bwd(st["qw"], st["ad"], self.X[p.d_in], self.dY[p.d_out], True, True, self.dX[p.d_in],
                             st["dA"], st["dB"], self.ws, saved=self.saved)
        if before_phase:
            before_phase("done")

    def merge_batch(self):
        qb, wl = self.qb, self.wl
        for st in self.proj:
            qb.qblora_tile_product(st["ad"], st["p"].d_in, st["p"].d_out, st["H"], self.ws)
        # all projections of the layer in one call (one launch where the kernels allow it)
        qb.qablora_merge_quantize_batch([st["qw"] for st in self.proj], [st["H"] for st in self.proj], self.lam, self.lam,
                                        wl.s, qb.MERGE_REQUANT_MINMAX, outs=[st["merged"] for st in self.proj])

    def step(self):
        for st in self.proj:
            self.layer_pass(st)
        self.merge_batch()

    # ---- counted work -------------------------------------------------------------------------------------
    def flops_step(self):
        T, r = self.T, self.rank
        return sum(4.0 * T * st["p"].d_in * st["p"].d_out + 6.0 * T * r * (st["p"].d_in + st["p"].d_out) for st in self.proj)

    def merge_bytes(self, p):
        lam = self.lam
        scale_in = (1 / 64 + 8 / (64 * 256)) if self.wl.scale_mode else 4 / 64
        return p.d_in * p.d_out * (0.5 + scale_in + 4.0 / (lam * lam) + 0.5 + 8 / 64)

    def describe(self):
        wl = self.wl
        shapes = {}
        for st in self.proj:
            k = f"{st['p'].d_out}x{st['p'].d_in}"
            shapes[k] = shapes.get(k, 0) + 1
        return (f"{wl.name}: T={self.T} tokens, projections " + " + ".join(f"{n} x [{k}]" for k, n in shapes.items()) +
                f", 4-bit block {wl.block}" + (" with double-quantized (E4M3, groups of 256) block scales" if wl.scale_mode else "") +
                f", adapter rank {self.rank}, lambda {self.lam} (inner rank {self.R}), s={wl.s}")


def stats(ms):
    import numpy as np
    a = np.asarray(ms, dtype=np.float64)
    return {"mean": round(float(a.mean()), 4), "median": round(float(np.median(a)), 4), "min": round(float(a.min()), 4)}


def measure(S, steps, warmup, side_steps, plain_events=False, calibration_copy=False):
    """Times `steps` steps of the workload held by `S` at its current rank; returns the result dict."""
    import numpy as np
    import torch
    from paper_2407_17029_amd import binding as qb

    wl, dev = S.wl, S.dev
    T, lam, R, r = S.T, S.lam, S.R, S.rank
    # the projection whose kernels are bracketed: the one with the most weights (first of equals)
    big = max(range(len(S.proj)), key=lambda i: (S.proj[i]["p"].d_in * S.proj[i]["p"].d_out, -i))
    bp = S.proj[big]["p"]

    if calibration_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 256 MiB, writes 256 MiB: a kernel of known traffic for counter runs
        torch.cuda.synchronize()
        del src, dst

    for _ in range(warmup):
        S.step()
    torch.cuda.synchronize()

    new_event = (lambda: torch.cuda.Event(enable_timing=True)) if plain_events else qb.TimingEvent
    # bench key -> (library slot, phase of the layer pass in which the pair is registered)
    slots = {"fwd_gemm": (qb.PROFILE_FWD_GEMM, "fwd"), "bwd_gemm": (qb.PROFILE_BWD_GEMM, "bwd"),
             "quantize": (qb.PROFILE_QUANTIZE, "quantize"),
             "adapter_fwd": (qb.PROFILE_ADAPTER_FWD, "fwd"), "adapter_bwd": (qb.PROFILE_ADAPTER_BWD, "bwd"),
             "adapter_grads": (qb.PROFILE_ADAPTER_GRADS, "bwd"), "grad_reduce": (qb.PROFILE_GRAD_REDUCE, "bwd"),
             "prep": (qb.PROFILE_PREP, "fwd"), "dequant_fwd": (qb.PROFILE_DEQUANT, "fwd"),
             "dequant_bwd": (qb.PROFILE_DEQUANT, "bwd"), "tile_product": (qb.PROFILE_TILE_PRODUCT, "merge"),
             "merge": (qb.PROFILE_MERGE, "merge")}
    dense = T >= qb.qblora_dense_min_tokens()           # the calls dequantize once, then contract the bf16 weight
    events = {k: [(new_event(), new_event()) for _ in range(steps if k == "fwd_gemm" else side_steps)] for k in slots}
    marks = [new_event() for _ in range(steps + 1)]
    for pairs in events.values():
        for a, b in pairs:
            a.record(); b.record()          # creates the native handles
    for m in marks:
        m.record()
    torch.cuda.synchronize()
    # What an event pair measures with nothing in between (the stream's cost of processing the second record);
    # taken off the bracketed GEMMs' elapsed times, which then agree with the kernel trace.
    empty_pair_ms = float(np.median([a.elapsed_time(b) for pairs in events.values() for a, b in pairs]))

    def bracketed_step(i, which):
        """One step with the event pairs of `which` registered around projection `big`'s calls only."""
        def hook(phase):
            for k in which:
                slot, ph = slots[k]
                if ph == "merge":
                    continue
                qb.qblora_profile_events(slot, None, None)
            for k in which:
                slot, ph = slots[k]
                if ph == phase:
                    qb.qblora_profile_events(slot, *events[k][i])

        for j, st in enumerate(S.proj):
            S.layer_pass(st, hook if j == big else None)
        # the merge batch: one pair around all tile products, one (registered with the library, so that it sits
        # directly around the launch) around the one launch that merges all projections
        if "merge" in which:
            events["tile_product"][i][0].record()
            for st in S.proj:
                qb.qblora_tile_product(st["ad"], st["p"].d_in, st["p"].d_out, st["H"], S.ws)
            events["tile_product"][i][1].record()
            qb.qblora_profile_events(qb.PROFILE_MERGE, *events["merge"][i])
            qb.qablora_merge_quantize_batch([st["qw"] for st in S.proj], [st["H"] for st in S.proj], lam, lam, wl.s,
                                            qb.MERGE_REQUANT_MINMAX, outs=[st["merged"] for st in S.proj])
            qb.qblora_profile_events(qb.PROFILE_MERGE, None, None)
        else:
            S.merge_batch()

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        marks[i].record()
        bracketed_step(i, ("fwd_gemm",))
    marks[steps].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    side = [k for k in slots if k != "fwd_gemm"]
    for i in range(side_steps):             # untimed: one event pair per kernel of the bracketed projection
        bracketed_step(i, side)
    torch.cuda.synchronize()

    raw = {k: [a.elapsed_time(b) for a, b in pairs] for k, pairs in events.items()}
    step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    ms_per_step = elapsed * 1e3 / steps
    flops_step = S.flops_step()
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    def gemm_ms(k):
        return max(float(np.mean(raw[k])) - empty_pair_ms, 1e-6)

    if not dense:                                       # no one-off dequantize pass in these calls
        raw["dequant_fwd"] = raw["dequant_bwd"] = [0.0]

    fwd_flops = 2.0 * T * bp.d_in * bp.d_out + 2.0 * T * R * bp.d_out / lam
    bwd_flops = 2.0 * T * bp.d_in * bp.d_out + 2.0 * T * R * bp.d_in / lam
    n_w = bp.d_in * bp.d_out
    quant_bytes = n_w * (4 + 0.5 + 4 / 64)
    merge_batch_bytes = sum(S.merge_bytes(st["p"]) for st in S.proj)
    achieved = fwd_flops / (gemm_ms("fwd_gemm") * 1e-3) / 1e12

    def hbm(k, nbytes, note=None):
        ms = float(np.mean(raw[k]))
        d = {"bound": "hbm", "event_overhead_included": True, "ms": stats(raw[k]),
             "achieved": round(nbytes / (ms * 1e-3) / 1e9, 1), "unit": "GB/s",
             "frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "algorithmic_bytes": int(nbytes)}
        if note:
            d["note"] = note
        if nbytes <= 256e6:                 # the launch's operands can stay in the 256 MB last-level cache from one
            d["fits_last_level_cache"] = True   # step to the next: then this is not a rate HBM delivered
        return d

    proj_name = f"{bp.name} [{bp.d_out}x{bp.d_in}]"
    kname = ("k_qlinear<0> (forward contraction on the weight dequantized once per call)" if dense
             else "k_qlinear<1> (forward dequantize-and-contract)")
    out = {
        "value": round(value, 2), "unit": "TFLOP/s", "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "step_ms": stats(step_ms),
        "tokens_per_s": round(T / (ms_per_step * 1e-3), 1),
        "pct_of_bf16_mfma_peak": round(100.0 * value / MFMA_BF16_PEAK_TFLOPS, 2),
        "workload": S.describe(), "counted_flops_per_step": flops_step,
        "roofline": {"kernel": kname, "projection": proj_name, "bound": "mfma",
                     "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": measured_traffic(wl.name, "fwd_gemm"),
                     "avg_kernel_ms": round(gemm_ms("fwd_gemm"), 4), "kernel_ms": stats(raw["fwd_gemm"]),
                     "empty_event_pair_ms": round(empty_pair_ms, 4), "algorithmic_flops": fwd_flops},
        "kernels": {
            "projection": proj_name,
            "bwd_gemm": {"bound": "mfma", "avg_kernel_ms": round(gemm_ms("bwd_gemm"), 4), "kernel_ms": stats(raw["bwd_gemm"]),
                         "achieved": round(bwd_flops / (gemm_ms("bwd_gemm") * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
                         "frac": round(bwd_flops / (gemm_ms("bwd_gemm") * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)},
            "quantize": hbm("quantize", quant_bytes),
            "dequantize_once_fwd": (hbm("dequant_fwd", n_w * (0.5 + 4 / 64 + 2), "codes + scales -> bf16 weight in the workspace")
                                    if dense else None),
            "dequantize_once_bwd": (hbm("dequant_bwd", n_w * (0.5 + 4 / 64 + 2), "the same, transposed, for the backward contraction")
                                    if dense else None),
            "adapter_fwd_skinny": hbm("adapter_fwd", 2.0 * T * bp.d_in + 2.0 * T * R * 2, "s*U = (s/lambda) X A_x^T; reads X once"),
            "adapter_bwd_skinny": hbm("adapter_bwd", 2.0 * T * bp.d_out + 2.0 * T * R * 3, "dU = s dY B_x^T; reads dY once"),
            "adapter_grads": hbm("adapter_grads", 2.0 * T * (bp.d_in + bp.d_out) + 8.0 * T * R,
                                 "token contractions behind dA and dB, one launch; partial-sum writes not counted"),
            "grad_reduce": {"ms": stats(raw["grad_reduce"])},
            "prep": {"ms": stats(raw["prep"])},
            "merge_requant_batch": hbm("merge", merge_batch_bytes,
                                       f"the requantizing merge of all {len(S.proj)} projections of the layer, one launch"),
            "tile_products": {"ms": stats(raw["tile_product"]),
                              "note": f"H = A B of all {len(S.proj)} projections, {len(S.proj)} launches back to back"},
        },
    }
    for k in ("quantize", "adapter_fwd", "adapter_bwd", "adapter_grads", "merge"):
        t = measured_traffic(wl.name, k)
        key = {"adapter_fwd": "adapter_fwd_skinny", "adapter_bwd": "adapter_bwd_skinny", "merge": "merge_requant_batch"}.get(k, k)
        out["kernels"][key]["traffic"] = t
    for k, key in (("quantize", "quantize"), ("merge", "merge_requant_batch"), ("dequant_fwd", "dequantize_once_fwd"),
                   ("dequant_bwd", "dequantize_once_bwd")):
        v = measured_valu(wl.name, k)
        if v and out["kernels"].get(key):
            out["kernels"][key].update(v)
    adapter_ms = sum(float(np.mean(raw[k])) for k in ("adapter_fwd", "adapter_bwd", "adapter_grads", "grad_reduce", "prep"))
    dq_ms = float(np.mean(raw["dequant_fwd"])) + float(np.mean(raw["dequant_bwd"]))
    proj_ms = adapter_ms + gemm_ms("fwd_gemm") + gemm_ms("bwd_gemm") + float(np.mean(raw["quantize"])) + dq_ms
    # the contraction with its share of the one-off dequantize pass, as one figure per direction
    for key, gk, dk, fl in (("fwd_gemm_with_dequantize", "fwd_gemm", "dequant_fwd", fwd_flops),
                            ("bwd_gemm_with_dequantize", "bwd_gemm", "dequant_bwd", bwd_flops)):
        ms = gemm_ms(gk) + float(np.mean(raw[dk]))
        out["kernels"][key] = {"ms": round(ms, 4), "achieved": round(fl / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
                               "frac": round(fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
    out["kernels"]["adapter_side_share_of_projection"] = round(adapter_ms / proj_ms, 4)
    return out


def cpu_baseline(S, sample_rows):
    """The fp64 oracle as it stands, on a bounded sample: for each distinct projection shape the one-off parts
    (quantize, dequantize, tile product, merge) in full and forward + backward on `sample_rows` token rows;
    extrapolated linearly in tokens and multiplied by how many projections have that shape."""
    import numpy as np
    import oracle
    from paper_2407_17029_amd import synth
    wl, T, lam, cb = S.wl, S.T, S.lam, S.cb
    ts = min(sample_rows, T)
    rows = synth.sample_rows(T, ts, wl.seed)
    seen = {}
    for i, st in enumerate(S.proj):
        p = st["p"]
        key = (p.d_out, p.d_in)
        if key in seen:
            seen[key]["count"] += 1
            continue
        W = S.host[("W", i)]
        A, B = S.host[("AB", i)]
        Xs = np.ascontiguousarray(S.host[("X", p.d_in)][rows])
        dYs = np.ascontiguousarray(S.host[("dY", p.d_out)][rows])
        c0 = time.perf_counter()
        codes, absmax = oracle.quantize_codebook(W, wl.block, cb)
        scales = absmax
        if wl.scale_mode:
            sc, stp, mid = oracle.scales_double_quantize(absmax.reshape(-1), 256)
            scales = oracle.scales_double_dequantize(sc, stp, mid, 256).reshape(absmax.shape)
        Wt = oracle.dequantize(codes, scales, None, cb, wl.block, 2)
        c1 = time.perf_counter()
        oracle.forward(Wt, Xs, A, B, lam, lam, wl.s)
        oracle.backward(Wt, Xs, dYs, A, B, lam, lam, wl.s)
        c2 = time.perf_counter()
        del Wt
        Ho = oracle.tile_product(A, B).astype(np.float32)
        oracle.merge_requant(codes, scales, None, cb, Ho, wl.block, lam, lam, wl.s)
        c3 = time.perf_counter()
        seen[key] = {"count": 1, "one_off": (c1 - c0) + (c3 - c2), "token_part": c2 - c1}
    measured = sum(v["one_off"] + v["token_part"] for v in seen.values())
    est_full = sum(v["count"] * (v["one_off"] + v["token_part"] * (T / ts)) for v in seen.values())
    return {"value": round(S.flops_step() / est_full / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.get_threads(),
            "kind": "oracle", "extrapolated": True,
            "sample": f"fp64 oracle, {measured:.1f} s measured: for each of the {len(seen)} distinct projection shapes the "
                      f"quantize + dequantize + tile product + merge in full and forward + backward (dX, dA, dB) on {ts} of {T} "
                      f"token rows; EXTRAPOLATED linearly in tokens (x{T / ts:.0f}) and by the number of projections of each "
                      f"shape to the full step: {est_full:.0f} s"}



# ---- side measurements: streaming kernels on the large layer shapes, and the rows next to the hot path -------
# Each entry: 10 warm-up launches, then 50 back-to-back launches between two HIP events on the current stream;
# `us` is with warm caches (the 256 MB last-level cache holds the operands of the smaller shapes between
# launches), `cold_us` rotates the launches over enough operand sets to exceed that cache, so that every launch
# reads from HBM.  The short kernels are launched through the C ABI with arguments marshalled once, so that the
# host keeps ahead of the GPU.
SHAPES = [(4096, 4096), (11008, 4096), (22016, 8192)]          # 7B attention, 7B MLP up, 65B MLP up
DEV = "cuda:0"


def timed(fn, iters=50, warm=10):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters * 1e-3                      # seconds per launch


def timed_rotating(fns, iters=50, warm=10):
    """Like timed(), the launches cycling through `fns` (one per operand set)."""
    n = len(fns)
    for i in range(warm):
        fns[i % n]()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(iters):
        fns[i % n]()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters * 1e-3


def n_sets(bytes_per_set, cache_bytes=256 * 2**20):
    """Operand sets needed so that a set has left the last-level cache when its turn comes again."""
    return max(2, int(np.ceil(2 * cache_bytes / max(bytes_per_set, 1))) + 1)


_SIDE = []


def emit(**kw):
    _SIDE.append(kw)


def bench_quantize():
    cb = synth.codebook_nf4_style()
    for d_out, d_in in SHAPES:
        W = torch.randn(d_out, d_in, device=DEV) * 0.02
        qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, cb, tiled=False)
        q, cbp = qw.c_struct(), np.ascontiguousarray(cb, np.float32)
        args = (qb._ptr(W), d_out, d_in, 64, qb.QUANT_ABSMAX_CODEBOOK, cbp.ctypes.data_as(C.c_void_p), qb.SCALES_FP32,
                C.byref(q), qb._stream())
        s = timed(lambda: qb.lib().qblora_quantize_blockwise(*args))
        nbytes = d_out * d_in * (4 + 0.5 + 4 / 64)
        # cold: every launch reads another copy of W
        Ws = [W] + [W.clone() for _ in range(n_sets(4 * d_out * d_in) - 1)]
        fns = []
        for Wi in Ws:
            ai = (qb._ptr(Wi),) + args[1:]
            fns.append(lambda ai=ai: qb.lib().qblora_quantize_blockwise(*ai))
        sc = timed_rotating(fns)
        emit(kernel="quantize_codebook", shape=[d_out, d_in], us=round(s * 1e6, 1), GBps=round(nbytes / s / 1e9, 1),
             frac_hbm=round(nbytes / s / 1e9 / HBM_PEAK_GBS, 3), cold_us=round(sc * 1e6, 1), cold_sets=len(Ws),
             cold_frac_hbm=round(nbytes / sc / 1e9 / HBM_PEAK_GBS, 3))
        del W, qw, Ws, fns


def bench_merge():
    cb = synth.codebook_nf4_style()
    for d_out, d_in in SHAPES:
        for lam in (2, 8):
            W = torch.randn(d_out, d_in, device=DEV) * 0.02
            qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, cb, tiled=False)
            H = torch.randn(d_in // lam, d_out // lam, device=DEV) * 0.01
            out = qb.qablora_merge_quantize(qw, H, lam, lam, 1.0, qb.MERGE_REQUANT_MINMAX)
            b, o = qw.c_struct(), out.c_struct()
            args = (C.byref(b), qb._ptr(H), lam, lam, C.c_float(1.0), qb.MERGE_REQUANT_MINMAX, C.byref(o), qb._stream())
            s = timed(lambda: qb.lib().qablora_merge_quantize(*args))
            nbytes = d_out * d_in * (0.5 + 4 / 64 + 4.0 / (lam * lam) + 0.5 + 8 / 64)
            # cold: every launch works on another copy of the weight, of H and of the output
            keep, fns = [], []
            for _ in range(n_sets(nbytes) - 1):
                qi = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, cb, tiled=False)
                Hi = H.clone()
                oi = qb.qablora_merge_quantize(qi, Hi, lam, lam, 1.0, qb.MERGE_REQUANT_MINMAX)
                bi, ooi = qi.c_struct(), oi.c_struct()
                ai = (C.byref(bi), qb._ptr(Hi), lam, lam, C.c_float(1.0), qb.MERGE_REQUANT_MINMAX, C.byref(ooi), qb._stream())
                keep.append((qi, Hi, oi, bi, ooi))
                fns.append(lambda ai=ai: qb.lib().qablora_merge_quantize(*ai))
            fns.append(lambda: qb.lib().qablora_merge_quantize(*args))
            sc = timed_rotating(fns)
            emit(kernel="merge_requant", shape=[d_out, d_in], lam=lam, us=round(s * 1e6, 1),
                 GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_PEAK_GBS, 3),
                 cold_us=round(sc * 1e6, 1), cold_sets=len(fns), cold_frac_hbm=round(nbytes / sc / 1e9 / HBM_PEAK_GBS, 3))
            del W, qw, H, out, keep, fns


def _decode_sets(d_out, d_in, **quant_kw):
    """Enough quantized copies (weight, pack, C struct) of one layer for the cold measurement."""
    wbytes = d_out * d_in * (0.5 + 8 / 64)
    sets = []
    for _ in range(n_sets(wbytes)):
        W = torch.randn(d_out, d_in, device=DEV) * 0.02
        qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_MINMAX_INT4, tiled=False, **quant_kw)
        sets.append((qw, qb.qblora_decode_pack(qw), qw.c_struct()))
        del W
    return sets


DECODE_SHAPES = SHAPES + [(8192, 8192), (8192, 22016)]            # + 65B attention and MLP down


def bench_decode():
    """`us`: one weight set, which the 256 MB last-level cache holds between launches (every shape here is smaller);
    `cold_us`: the launches rotate over enough sets that each reads its weights from HBM, as inference over the
    layers of a model does.  frac_hbm / cold_frac_hbm = the weight stream's bytes over those times."""
    for d_out, d_in in DECODE_SHAPES:
        sets = _decode_sets(d_out, d_in)
        qw, pack, qp = sets[0]
        sp = timed(lambda: qb.lib().qblora_decode_pack(C.byref(qp), qb._ptr(pack), qb._stream()), iters=10, warm=2)
        emit(kernel="decode_pack (one-off)", shape=[d_out, d_in], us=round(sp * 1e6, 1))
        for T in (1, 2, 4, 8, 16):
            X = torch.randn(T, d_in, device=DEV).to(torch.bfloat16)
            Y = torch.empty(T, d_out, dtype=torch.bfloat16, device=DEV)
            for name in ("packed", "row-major"):
                if name == "row-major" and (T not in (1, 16) or (d_out, d_in) not in SHAPES):
                    continue
                fns = []
                for qi, pk, ci in sets:
                    ai = (C.byref(ci), qb._ptr(pk if name == "packed" else None), qb._ptr(X), T, qb._ptr(Y), None, 0,
                          qb._stream())
                    fns.append(lambda ai=ai: qb.lib().qblora_linear_decode(*ai))
                s = timed(fns[0], iters=50)
                sc = timed_rotating(fns, iters=60, warm=12)
                nbytes = d_out * d_in * (0.5 + 8 / 64) + 2 * T * (d_in + d_out)
                emit(kernel="w4_decode", layout=name, shape=[d_out, d_in], T=T, us=round(s * 1e6, 1),
                     GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_PEAK_GBS, 3),
                     cold_us=round(sc * 1e6, 1), cold_sets=len(fns),
                     cold_frac_hbm=round(nbytes / sc / 1e9 / HBM_PEAK_GBS, 3))
        del sets, qw, pack


def bench_midbatch():
    """16 < T <= 256 on the merged INT4 model (packed) and on a codebook base (row-major): time against the two
    floors of the regime, the weight stream from HBM and the bf16 MFMA work.  `us` with one weight set (held by the
    last-level cache between launches), `cold_us` rotating over sets so that the weights come from HBM."""
    cb = synth.codebook_nf4_style()
    for d_out, d_in in SHAPES:
        for base in ("int4 packed", "codebook row-major"):
            sets = []
            for _ in range(n_sets(d_out * d_in * 0.625)):
                W = torch.randn(d_out, d_in, device=DEV) * 0.02
                if base == "int4 packed":
                    qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_MINMAX_INT4, tiled=False)
                    sets.append((qw, qb.qblora_decode_pack(qw), qw.c_struct()))
                else:
                    qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, cb, tiled=False)
                    sets.append((qw, None, qw.c_struct()))
                del W
            qw, q = sets[0][0], sets[0][2]
            for T in (32, 64, 128, 256):
                X = torch.randn(T, d_in, device=DEV).to(torch.bfloat16)
                Y = torch.empty(T, d_out, dtype=torch.bfloat16, device=DEV)
                need = int(qb.lib().qblora_linear_decode_tokens_workspace_bytes(C.byref(q), T))
                ws = torch.empty(max(need, 256), dtype=torch.uint8, device=DEV)
                fns = []
                for qi, pk, ci in sets:
                    ai = (C.byref(ci), qb._ptr(pk), qb._ptr(X), T, qb._ptr(Y), qb._ptr(ws), ws.numel(), qb._stream())
                    fns.append(lambda ai=ai: qb.lib().qblora_linear_decode(*ai))
                s = timed(fns[0], iters=30)
                sc = timed_rotating(fns, iters=36, warm=len(fns))
                nbytes = d_out * d_in * (0.5 + (8 if qw.beta is not None else 4) / 64) + 2 * T * (d_in + d_out)
                flops = 2.0 * T * d_in * d_out
                emit(kernel="w4_mid", base=base, shape=[d_out, d_in], T=T, us=round(s * 1e6, 1),
                     GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_PEAK_GBS, 3),
                     cold_us=round(sc * 1e6, 1), cold_sets=len(fns),
                     cold_frac_hbm=round(nbytes / sc / 1e9 / HBM_PEAK_GBS, 3),
                     TFLOPs=round(flops / s / 1e12, 1), frac_mfma=round(flops / s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 3),
                     partial_bytes=need)
            del sets, qw


def bench_qablora():
    cb = synth.codebook_nf4_style()
    T, d_out, d_in = 8192, 4096, 4096
    W = torch.randn(d_out, d_in, device=DEV) * 0.02
    qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_ABSMAX_CODEBOOK, cb)
    X = torch.randn(T, d_in, device=DEV).to(torch.bfloat16)
    dY = torch.randn(T, d_out, device=DEV).to(torch.bfloat16)
    Y = torch.empty_like(dY)
    dX = torch.empty_like(X)
    for l1, l2 in ((8, 8), (4, 8), (2, 2)):
        H = (torch.randn(d_in // l1, d_out // l2, device=DEV) * 0.02).to(torch.bfloat16)
        dH = torch.empty(d_in // l1, d_out // l2, device=DEV)
        f = timed(lambda: qb.qablora_linear_fwd(qw, H, l1, l2, 1.0, X, Y), iters=10)
        b = timed(lambda: qb.qablora_linear_bwd(qw, H, l1, l2, 1.0, X, dY, True, True, dX, dH), iters=10)
        flops = 4.0 * T * d_in * d_out + 6.0 * T * (d_in // l1) * (d_out // l2)
        emit(kernel="qablora_fwd+bwd", shape=[d_out, d_in], T=T, lam=[l1, l2], fwd_us=round(f * 1e6, 1),
             bwd_us=round(b * 1e6, 1), TFLOPs=round(flops / (f + b) / 1e12, 1),
             frac_mfma=round(flops / (f + b) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 3))


def bench_tile8():
    """The quantization-aware loop on 8 x 8 quantization blocks (block 64 with lambda1 = lambda2 = 8): min-max INT4
    quantizer, single-matrix forward / backward, the exact offset-shift merge, small-batch inference."""
    T, d_out, d_in, l1, l2 = 8192, 4096, 4096, 8, 8
    W = torch.randn(d_out, d_in, device=DEV) * 0.02
    qw = qb.qblora_quantize_blockwise(W, 64, qb.QUANT_MINMAX_INT4, block_rows=8, tiled=True)
    q = qw.c_struct()
    args = (qb._ptr(W), d_out, d_in, 64, qb.QUANT_MINMAX_INT4, None, qb.SCALES_FP32, C.byref(q), qb._stream())
    s = timed(lambda: qb.lib().qblora_quantize_blockwise(*args))
    nbytes = d_out * d_in * (4 + 0.5 + 8 / 64)
    emit(kernel="quantize_minmax 8x8 blocks (+ tile-ordered code copy)", shape=[d_out, d_in], us=round(s * 1e6, 1),
         GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_PEAK_GBS, 3))
    X = torch.randn(T, d_in, device=DEV).to(torch.bfloat16)
    dY = torch.randn(T, d_out, device=DEV).to(torch.bfloat16)
    Y = torch.empty_like(dY)
    dX = torch.empty_like(X)
    H = (torch.randn(d_in // l1, d_out // l2, device=DEV) * 0.02).to(torch.bfloat16)
    dH = torch.empty(d_in // l1, d_out // l2, device=DEV)
    f = timed(lambda: qb.qablora_linear_fwd(qw, H, l1, l2, 1.0, X, Y), iters=10)
    b = timed(lambda: qb.qablora_linear_bwd(qw, H, l1, l2, 1.0, X, dY, True, True, dX, dH), iters=10)
    flops = 4.0 * T * d_in * d_out + 6.0 * T * (d_in // l1) * (d_out // l2)
    emit(kernel="qablora_fwd+bwd 8x8 blocks", shape=[d_out, d_in], T=T, lam=[l1, l2], fwd_us=round(f * 1e6, 1),
         bwd_us=round(b * 1e6, 1), TFLOPs=round(flops / (f + b) / 1e12, 1),
         frac_mfma=round(flops / (f + b) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 3))
    Hf = H.float().contiguous()
    merged = qb.qablora_merge_quantize(qw, Hf, l1, l2, 1.0, qb.MERGE_BETA_SHIFT)
    bq, o = qw.c_struct(), merged.c_struct()
    margs = (C.byref(bq), qb._ptr(Hf), l1, l2, C.c_float(1.0), qb.MERGE_BETA_SHIFT, C.byref(o), qb._stream())
    s = timed(lambda: qb.lib().qablora_merge_quantize(*margs))
    nb = d_out * d_in // 64
    nbytes = d_out * d_in * 0.5 * 2 + nb * 4 * 4 + Hf.numel() * 4           # codes and alpha copied, beta shifted
    emit(kernel="merge_beta_shift 8x8 blocks (codes + alpha copied)", shape=[d_out, d_in], us=round(s * 1e6, 1),
         GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_PEAK_GBS, 3))
    for d_out2, d_in2 in ((4096, 4096), (22016, 8192)):
        sets = _decode_sets(d_out2, d_in2, block_rows=8)
        for Tn in (1, 4, 16):
            Xs = torch.randn(Tn, d_in2, device=DEV).to(torch.bfloat16)
            Ys = torch.empty(Tn, d_out2, dtype=torch.bfloat16, device=DEV)
            fns = []
            for qi, pk, ci in sets:
                ai = (C.byref(ci), qb._ptr(pk), qb._ptr(Xs), Tn, qb._ptr(Ys), None, 0, qb._stream())
                fns.append(lambda ai=ai: qb.lib().qblora_linear_decode(*ai))
            s = timed(fns[0], iters=50)
            sc = timed_rotating(fns, iters=60, warm=12)
            nbytes = d_out2 * d_in2 * (0.5 + 8 / 64) + 2 * Tn * (d_in2 + d_out2)
            emit(kernel="w4_decode 8x8 blocks", layout="packed", shape=[d_out2, d_in2], T=Tn, us=round(s * 1e6, 1),
                 GBps=round(nbytes / s / 1e9, 1), frac_hbm=round(nbytes / s / 1e9 / HBM_PEAK_GBS, 3),
                 cold_us=round(sc * 1e6, 1), cold_sets=len(fns),
                 cold_frac_hbm=round(nbytes / sc / 1e9 / HBM_PEAK_GBS, 3))
        del sets


def side_measurements(which):
    import ctypes, numpy, torch
    from paper_2407_17029_amd import binding, synth as synth_mod
    g = globals()
    g.update(C=ctypes, np=numpy, torch=torch, qb=binding, synth=synth_mod)
    del _SIDE[:]
    table = {"quantize": bench_quantize, "merge": bench_merge, "decode": bench_decode, "midbatch": bench_midbatch,
             "qablora": bench_qablora,
             "tile8": bench_tile8}
    for w in which:
        table[w]()
        torch.cuda.empty_cache()
    return list(_SIDE)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama65b_layer")
    ap.add_argument("--rank", type=int, default=0, help="adapter rank D_rank (0 = the workload's own)")
    ap.add_argument("--cpu-sample-rows", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the other workloads (the `configs` object)")
    ap.add_argument("--side", default="quantize,merge,decode,midbatch,qablora,tile8",
                    help="comma-separated side measurements reported under `side` (streaming kernels on the large shapes, "
                         "small-batch inference, single-matrix adapter, 8 x 8 blocks); empty string = none")
    ap.add_argument("--plain-events", action="store_true",
                    help="time the kernels with ordinary HIP events (system-scope fence at every record)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of 256 MiB before the timed steps, so that a counter "
                         "profile of this command holds a kernel of known traffic to scale FETCH_SIZE/WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (no collectives are part of it); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2407_17029_amd import binding as qb
    from paper_2407_17029_amd import synth

    dev = "cuda:0"
    torch.cuda.set_device(0)
    qb.lib()
    side_steps = max(1, min(args.steps, 5))
    wl = synth.WORKLOADS[args.workload]
    S = Stack(wl, args.rank or wl.rank, dev)
    res = measure(S, args.steps, args.warmup, side_steps, args.plain_events, args.calibration_copy)
    out = {
        "metric": "fused quantized-linear+BLoRA fwd+bwd TFLOP/s",
        "value": res["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": res["workload"],
                   "step": "per projection: quantize + forward + backward(dX,dA,dB); then tile product + INT4 requantizing "
                           "merge of all projections"},
        "step_ms": res["step_ms"], "tokens_per_s": res["tokens_per_s"],
        "pct_of_bf16_mfma_peak": res["pct_of_bf16_mfma_peak"],
        "roofline": res["roofline"], "kernels": res["kernels"],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(S, args.cpu_sample_rows)
    del S
    torch.cuda.empty_cache()

    if not args.no_configs:
        cfg = {}
        others = [n for n in ("llama7b_attn", "llama7b_mlp", "llama13b_layer") if n != args.workload]
        for name in others:
            steps = max(3, min(args.steps, 10))
            wl2 = synth.WORKLOADS[name]
            S2 = Stack(wl2, wl2.rank, dev)
            r = measure(S2, steps, 3, min(3, side_steps), args.plain_events)
            entry = {k: r[k] for k in ("value", "unit", "steps", "ms_per_step", "step_ms", "tokens_per_s",
                                       "pct_of_bf16_mfma_peak", "workload")}
            entry["roofline"] = {k: r["roofline"][k] for k in ("kernel", "projection", "bound", "achieved", "peak", "unit",
                                                               "frac", "traffic", "avg_kernel_ms")}
            entry["kernels"] = {"bwd_gemm_frac": r["kernels"]["bwd_gemm"]["frac"],
                                "quantize_frac": r["kernels"]["quantize"]["frac"],
                                "merge_requant_batch_frac": r["kernels"]["merge_requant_batch"]["frac"],
                                "merge_requant_batch_fits_last_level_cache":
                                    r["kernels"]["merge_requant_batch"].get("fits_last_level_cache", False),
                                "adapter_side_share_of_projection": r["kernels"]["adapter_side_share_of_projection"]}
            if name == "llama13b_layer":
                sweep = {str(wl2.rank): {"value": r["value"], "ms_per_step": r["ms_per_step"],
                                         "roofline_frac": r["roofline"]["frac"]}}
                for rk in (32, 128):
                    S2.set_rank(rk)
                    rr = measure(S2, steps, 3, 1, args.plain_events)
                    sweep[str(rk)] = {"value": rr["value"], "ms_per_step": rr["ms_per_step"],
                                      "roofline_frac": rr["roofline"]["frac"]}
                entry["rank_sweep"] = sweep
            del S2
            torch.cuda.empty_cache()
            cfg[name] = entry
        out["configs"] = cfg
    side = [w for w in args.side.split(",") if w]
    if side:
        out["side"] = side_measurements(side)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
