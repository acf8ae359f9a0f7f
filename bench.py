#!/usr/bin/env python3
"""Benchmark of the Dynamic Mask Attention hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch already resident in HBM:
dma_mask_gen (scores, top-k expiry, slot plan) + dma_fwd + dma_bwd, all through the C ABI.
Prints ONE JSON line.  `value` is the effective TFLOP/s of the step: the algorithmic
forward+backward FLOPs (14 * d per kept (query, key) pair) divided by the step time, mask
generation included.  `roofline` is measured live with HIP events recorded inside the library
around each kernel stage; `cpu_baseline` times the CPU oracle on a bounded sample.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16, published
HBM_PEAK_GBS = 8000.0               # MI355X HBM3E, published
HEADLINE = "cfg3"


def n_active(seqlens, k):
    tot = 0
    for n in seqlens:
        n = int(n)
        tot += n * (n + 1) // 2 if k >= n else k * n - k * (k - 1) // 2
    return tot


class HipEvents:
    """Raw hipEvent_t handles (the library records them; torch's events wrap the same API)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.arr = (ctypes.c_void_p * n)()
        for i in range(n):
            ev = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(ev))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            self.arr[i] = ev

    def elapsed(self, i, j):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.arr[i], self.arr[j])
        return ms.value if rc == 0 else float("nan")

    def destroy(self):
        for ev in self.arr:
            self.hip.hipEventDestroy(ev)


def cpu_baseline(inp, wl, flops_per_head):
    """The oracle as it stands, on the q-heads of one kv-group of the same workload."""
    import oracle as orc
    G = wl.H_q // wl.H_kv
    nh = min(G, 4)
    Q, K, V, dO = inp.Q[:, :nh], inp.K[:, :1], inp.V[:, :1], inp.dO[:, :nh]
    t0 = time.perf_counter()
    z = orc.z_scores(V, inp.W[:nh], inp.A[:nh], nh)
    orc.dma_forward(Q, K, V, z, inp.cu_seqlens, wl.k)
    if wl.backward:
        orc.dma_backward(Q, K, V, z, dO, inp.cu_seqlens, wl.k)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": nh * flops_per_head / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{nh} of {wl.H_q} q-heads (one kv-head) of {wl.name}, all rows, scores + forward"
                      f"{' + backward' if wl.backward else ''}, {dt:.1f} s; same algorithmic FLOPs per head",
            "seconds": dt}


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` at the headline shape, from the committed rocprofv3 counter
    summary (FETCH_SIZE / WRITE_SIZE runs scaled by a copy of known size); None if not recorded."""
    path = os.path.join(ROOT, "profiles", "hotpath_cfg3_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                cols = line.split()
                if cols and cols[0] == kernel and cols[-1].isdigit():
                    return int(cols[-1])
    except OSError:
        pass
    return None


def clean_pair_count(inp, eg, BQ=256):
    """Kept (row, key) pairs whose key is resident for ALL rows of the pair's 256-row block (the pairs
    dkv_kernel<clean> works on), summed over heads; counted on the host from the expiry array."""
    import numpy as np
    clean_pairs = 0
    for a, b in zip(inp.cu_seqlens[:-1], inp.cu_seqlens[1:]):
        a, b = int(a), int(b)
        n = b - a
        if n == 0:
            continue
        j = np.arange(n)[None, :]
        e = eg[:, a:b] - a
        first = j // BQ + 1                                   # first block a key can be clean in
        # block bl is clean for the key iff bl >= first and e > min((bl + 1) BQ, n) - 1
        last_full = np.where(e >= n, (n - 1) // BQ, e // BQ - 1)    # last block with e > its last row
        nb = np.clip(last_full - first + 1, 0, None) * (e > j)
        rows_last = n - ((n - 1) // BQ) * BQ                  # rows of the (possibly ragged) last block
        pairs = nb * BQ - np.where((nb > 0) & (last_full == (n - 1) // BQ), BQ - rows_last, 0)
        clean_pairs += int(pairs.sum())
    return clean_pairs


def time_workload(wl, steps, warmup, dev, structured_z=False, calibration_copy=False):
    """Times `steps` steps (mask_gen + fwd [+ bwd]) of one workload.  Returns the timing record and the
    device case.  Stage events are recorded inside the timed region on every fourth step (an armed
    step records 20 events between the launches, 0.05-0.15 ms of a 3.3 ms step; the kernels'
    durations do not depend on it); per-step durations come from one event per step boundary."""
    import numpy as np
    import torch
    from paper_2508_02124_amd import binding as B
    from paper_2508_02124_amd import workloads as wlmod
    from paper_2508_02124_amd.device_case import DeviceCase
    inp = wlmod.make_inputs(wl)
    z_override = None
    if structured_z:
        rz = np.random.default_rng(wl.seed + 7)
        z_override = rz.uniform(0.05, 1.0, size=(wl.H_q, inp.T)).astype(np.float32)
        z_override[0::2] = (0.05 + 0.95 * (np.arange(inp.T, dtype=np.float64) + 1) / inp.T).astype(np.float32)[None, :]
    case = DeviceCase(inp, dev, z_override=z_override)
    seqlens = np.diff(inp.cu_seqlens)
    nact = n_active(seqlens, wl.k)
    per_pair = 14 if wl.backward else 4
    flops = float(per_pair) * wl.d * nact * wl.H_q

    def step():
        case.mask_gen()
        case.fwd()
        if wl.backward:
            case.bwd()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 256 MiB, writes 256 MiB: the yardstick for the HBM byte counters
        torch.cuda.synchronize()
        del src, dst

    nst = len(B.STAGES)
    armed = [i for i in range(steps) if i % 4 == 0]
    evsets = [HipEvents(2 * nst) for _ in armed]
    bounds = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    bounds[0].record()
    for i in range(steps):
        B.dma_profile_events(evsets[armed.index(i)].arr if i in armed else None)
        step()
        bounds[i + 1].record()
    B.dma_profile_events(None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    step_ms = [bounds[i].elapsed_time(bounds[i + 1]) for i in range(steps)]

    used = [s for s in range(nst) if wl.backward or s <= 4]
    samples = {B.STAGES[s]: [e.elapsed(2 * s, 2 * s + 1) for e in evsets] for s in used}
    for e in evsets:
        e.destroy()
    rec = {
        "ms_per_step": ms_per_step,
        "step_ms_median": float(np.median(step_ms)), "step_ms_min": float(np.min(step_ms)),
        "stage_ms": {n: float(np.mean(v)) for n, v in samples.items()},
        "stage_ms_median": {n: float(np.median(v)) for n, v in samples.items()},
        "stage_ms_min": {n: float(np.min(v)) for n, v in samples.items()},
        "flops": flops, "nact": int(nact), "seqlens": seqlens,
    }
    st = rec["stage_ms"]
    rec["mask_gen_ms"] = sum(st[n] for n in ("z", "sort", "expiry", "plan"))
    rec["fwd_ms"] = st["fwd"]
    rec["bwd_ms"] = sum(v for n, v in st.items() if n.startswith("bwd")) if wl.backward else 0.0
    return rec, case, inp


def roofline_objects(wl, inp, case, rec, with_traffic):
    """Roofline records of the kernels of the step.  MFMA kernels: algorithmic FLOPs of the launch
    (per kept pair: forward 4d = S and PV; dQ kernel 6d = S, dP, dQ; key-stationary kernel 8d = S, dP,
    dV, dK on the pairs of its launch) / mean launch duration / 2.5 PFLOP/s.  The score kernel of
    mask generation is HBM-bound: bytes of V read once + z and z / scale written, / duration / 8 TB/s
    (its stage also holds the block-table launch, a few microseconds)."""
    import numpy as np
    stage_ms = rec["stage_ms"]
    nact = rec["nact"]
    stage_flops = {"fwd": 4.0 * wl.d * nact * wl.H_q}
    if wl.backward:
        eg = case.host("expiry").astype(np.int64)
        stage_flops["bwd_dq"] = 6.0 * wl.d * nact * wl.H_q
        stage_flops["bwd_dkv"] = 8.0 * wl.d * clean_pair_count(inp, eg)
    kernel_names = {"fwd": "fwd_kernel", "bwd_dq": "dq_kernel", "bwd_dkv": "dkv_kernel<clean>"}
    objs = {}
    for st, fl in stage_flops.items():
        achieved = fl / (stage_ms[st] * 1e-3) / 1e12
        objs[kernel_names[st]] = {
            "bound": "mfma", "kernel": kernel_names[st], "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
            "traffic": measured_traffic(kernel_names[st]) if with_traffic else None,
            "launch_ms": stage_ms[st], "launch_ms_median": rec["stage_ms_median"][st],
            "launch_ms_min": rec["stage_ms_min"][st], "flops_per_launch": fl}
    zbytes = inp.T * wl.H_kv * wl.d * 2 + 2 * 4 * wl.H_q * inp.T
    zach = zbytes / (stage_ms["z"] * 1e-3) / 1e9
    objs["z_kernel"] = {"bound": "hbm", "kernel": "z_kernel (mask generation, Eq. 3)", "achieved": zach,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": zach / HBM_PEAK_GBS,
                        "traffic": measured_traffic("z_kernel") if with_traffic else None,
                        "launch_ms": stage_ms["z"], "launch_ms_median": rec["stage_ms_median"]["z"],
                        "launch_ms_min": rec["stage_ms_min"]["z"], "bytes_per_launch": zbytes}
    dom = max(stage_flops, key=lambda n: stage_ms[n])
    return kernel_names[dom], objs


SWEEP = [("cfg2", 0), ("cfg5", 0), ("cfg3", 512), ("cfg3", 1024), ("cfg3", 0), ("cfg3_d256", 0),
         ("cfg4", 1024), ("cfg4", 4096), ("cfg4", 16384), ("cfg4", 65536)]


def run_sweep(args, dev):
    """The benchmark spec's other shapes and the mask-density sweep of cfg4 (forward only), one record each:
    time must follow the number of kept pairs (k L - k^2 / 2 per head), not L^2."""
    import torch
    from paper_2508_02124_amd import workloads as wlmod
    rows = []
    for name, k in SWEEP:
        wl = wlmod.CONFIGS[name]
        if k:
            wl = wl.with_k(k)
        steps = max(3, min(args.steps, 10 if name == "cfg4" else args.steps))
        rec, case, inp = time_workload(wl, steps, args.warmup, dev)
        kname, objs = roofline_objects(wl, inp, case, rec, False)
        rows.append({
            "workload": f"{wl.name}: T={inp.T} docs={len(rec['seqlens'])} H_q={wl.H_q} H_kv={wl.H_kv} d={wl.d} k={wl.k} "
                        f"{'fwd+bwd' if wl.backward else 'fwd'}",
            "kept_pairs_all_heads": rec["nact"] * wl.H_q, "steps": steps,
            "ms_per_step": rec["ms_per_step"], "step_ms_median": rec["step_ms_median"], "step_ms_min": rec["step_ms_min"],
            "mask_gen_ms": rec["mask_gen_ms"], "fwd_ms": rec["fwd_ms"], "bwd_ms": rec["bwd_ms"],
            "stage_ms": rec["stage_ms"],
            "effective_tflops": rec["flops"] / (rec["ms_per_step"] * 1e-3) / 1e12,
            "fwd_kernel_tflops": objs["fwd_kernel"]["achieved"],
            "ns_per_kept_pair_fwd": rec["fwd_ms"] * 1e6 / (rec["nact"] * wl.H_q),
        })
        print(f"[sweep] {rows[-1]['workload']}: {rows[-1]['ms_per_step']:.3f} ms/step, fwd {rows[-1]['fwd_ms']:.3f} ms",
              file=sys.stderr, flush=True)
        del case, inp
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "dma_shape_sweep", "unit": "ms", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                      "sweep": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default=HEADLINE, help="cfg1..cfg5 or cfg3_d256 (default: the headline shape)")
    ap.add_argument("--k", type=int, default=0, help="override the keep-window (cfg4 sweep)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline line: cfg2, cfg5, cfg3 at k = 512 / 1024 / 2048 and the cfg4 "
                         "mask-density sweep k = 1K / 4K / 16K / 64K, one record each in one JSON line")
    ap.add_argument("--structured-z", action="store_true",
                    help="reported-only variant: scores supplied by the caller, even heads increasing with the "
                         "key index (a local band: each row keeps its k latest keys), odd heads i.i.d.")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2508_02124_amd import binding as B
    from paper_2508_02124_amd import probe as P
    from paper_2508_02124_amd import workloads as wlmod

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    if args.sweep:
        run_sweep(args, dev)
        return
    wl = wlmod.CONFIGS[args.config]
    if args.k:
        wl = wl.with_k(args.k)
    rec, case, inp = time_workload(wl, args.steps, args.warmup, dev, args.structured_z, args.calibration_copy)
    ms_per_step, stage_ms, flops, nact, seqlens = rec["ms_per_step"], rec["stage_ms"], rec["flops"], rec["nact"], rec["seqlens"]
    mask_ms, fwd_ms, bwd_ms = rec["mask_gen_ms"], rec["fwd_ms"], rec["bwd_ms"]
    dom_kernel, rooflines = roofline_objects(wl, inp, case, rec, wl.name == HEADLINE and not args.k)
    roofline = rooflines[dom_kernel]

    value = flops / (ms_per_step * 1e-3) / 1e12

    # yardsticks measured on this device: the MFMA rate from registers and a streaming copy
    prop = torch.cuda.get_device_properties(0)
    ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    nwg, iters = 4 * prop.multi_processor_count, 4096
    sink = torch.empty(nwg * 512, device=dev)
    P.dma_probe_mfma(sink, nwg, 64)
    best = float("inf")
    for _ in range(3):                                   # best of three 4 ms runs (the clock ramps up)
        ev2[0].record()
        P.dma_probe_mfma(sink, nwg, iters)
        ev2[1].record()
        torch.cuda.synchronize()
        best = min(best, ev2[0].elapsed_time(ev2[1]))
    mfma_measured = nwg * 8 * iters * 8 * 32768.0 / (best * 1e-3) / 1e12
    cbytes = 1 << 30
    csrc = torch.empty(cbytes, dtype=torch.uint8, device=dev).fill_(3)
    cdst = torch.empty_like(csrc)
    P.dma_probe_copy(csrc, cdst, cbytes)
    best = float("inf")
    for _ in range(3):
        ev2[0].record()
        P.dma_probe_copy(csrc, cdst, cbytes)
        ev2[1].record()
        torch.cuda.synchronize()
        best = min(best, ev2[0].elapsed_time(ev2[1]))
    copy_measured = 2.0 * cbytes / (best * 1e-3) / 1e9
    del csrc, cdst, sink
    device = {"name": prop.name or getattr(prop, "gcnArchName", ""), "compute_units": int(prop.multi_processor_count),
              "mfma_bf16_measured_tflops": mfma_measured, "stream_copy_measured_GB/s": copy_measured}
    out = {
        "metric": "dma_mask_fwd_bwd_effective_tflops" if wl.backward else "dma_mask_fwd_effective_tflops",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: T={inp.T} docs={len(seqlens)} H_q={wl.H_q} H_kv={wl.H_kv} d={wl.d} "
                               f"k={wl.k} causal bf16 {'fwd+bwd' if wl.backward else 'fwd'}"
                               f"{' structured-z' if args.structured_z else ''}",
                   "max_seqlen": int(inp.max_seqlen), "active_pairs_per_head": int(nact)},
        "pct_mfma_peak": 100.0 * value / MFMA_BF16_PEAK_TFLOPS,
        "pct_mfma_measured": 100.0 * value / mfma_measured, "device": device,
        "mask_gen_ms": mask_ms, "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "fwd_bwd_ms": fwd_ms + bwd_ms,
        "fwd_bwd_tflops": flops / ((fwd_ms + bwd_ms) * 1e-3) / 1e12,
        "step_ms_median": rec["step_ms_median"], "step_ms_min": rec["step_ms_min"],
        "stage_ms": stage_ms, "stage_ms_median": rec["stage_ms_median"], "stage_ms_min": rec["stage_ms_min"],
        "algorithmic_gflop": flops / 1e9,
        "roofline": roofline,
        "rooflines": rooflines,
    }
    if wl.backward:
        # not part of the step: the gradient of the content scores (dz -> dW, dA, dV += dVz), HBM-bound
        dW = torch.empty((wl.H_q, wl.d), device=dev)
        dA = torch.empty((wl.H_q,), device=dev)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
        B.dma_mask_bwd(case.shape, case.V, case.W, case.A, case.dz, dW, dA, case.dV, True)
        for i in range(5):
            ev[i].record()
            B.dma_mask_bwd(case.shape, case.V, case.W, case.A, case.dz, dW, dA, case.dV, True)
        ev[5].record()
        torch.cuda.synchronize()
        mb_ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(5)]))
        mb_bytes = 3 * inp.T * wl.H_kv * wl.d * 2 + 4 * wl.H_q * inp.T   # V read, dV read + write, dz read
        out["mask_bwd"] = {"ms": mb_ms, "algorithmic_bytes": mb_bytes, "GB/s": mb_bytes / (mb_ms * 1e-3) / 1e9,
                           "hbm_peak_GB/s": 8000.0}
        # not part of the step: the scores from the full cross-head Delta (Eq. 3) and their chain rule
        if wl.H_q <= 32 and wl.d <= 128:     # (the cross-head kernels take head dimensions 64 and 128)
            Dl = torch.randn((wl.H_q, wl.H_kv * wl.d), device=dev) / float(np.sqrt(wl.H_kv * wl.d))
            dDl = torch.empty_like(Dl)
            zx = torch.empty_like(case.z)
            times = {}
            for nm, fn in (("fwd", lambda: B.dma_scores_xhead(case.shape, case.V, Dl, case.A, zx)),
                           ("bwd", lambda: B.dma_scores_xhead_bwd(case.shape, case.V, Dl, case.A, case.dz, dDl, dA,
                                                                  case.dV, True))):
                fn()
                for i in range(5):
                    ev[i].record()
                    fn()
                ev[5].record()
                torch.cuda.synchronize()
                times[nm] = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(5)]))
            vb = inp.T * wl.H_kv * wl.d * 2
            out["scores_xhead"] = {"fwd_ms": times["fwd"], "fwd_algorithmic_bytes": vb + 4 * wl.H_q * inp.T,
                                   "bwd_ms": times["bwd"], "bwd_algorithmic_bytes": 3 * vb + 4 * wl.H_q * inp.T,
                                   "gflop_fwd": 2.0 * inp.T * wl.H_kv * wl.d * wl.H_q / 1e9}
    if wl.name == HEADLINE and not args.k:
        # not part of the step: decode of one new row against a 65536-token cache (HBM-bound)
        Ld, kd = 65536, 2048
        dshape = B.make_shape(T=Ld, n_docs=1, H_q=wl.H_q, H_kv=wl.H_kv, d=wl.d, k=kd)
        g = torch.Generator(device=dev).manual_seed(5)
        Kc = torch.randn((Ld, wl.H_kv, wl.d), device=dev, generator=g).to(torch.bfloat16)
        Vc = torch.randn((Ld, wl.H_kv, wl.d), device=dev, generator=g).to(torch.bfloat16)
        qc = torch.randn((1, wl.H_q, wl.d), device=dev, generator=g).to(torch.bfloat16)
        zc = torch.rand((wl.H_q, Ld), device=dev, generator=g)
        cuc = torch.tensor([0, Ld], dtype=torch.int32, device=dev)
        oc = torch.empty_like(qc)
        lc = torch.empty((wl.H_q, 1), device=dev)
        kb = B.dma_decode_kept_bytes(dshape)
        kc = torch.empty(kb // 4, dtype=torch.int32, device=dev)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
        B.dma_decode(dshape, qc, Kc, Vc, zc, cuc, oc, lc, kc, kb)
        for i in range(5):
            ev[i].record()
            B.dma_decode(dshape, qc, Kc, Vc, zc, cuc, oc, lc, kc, kb)
        ev[5].record()
        torch.cuda.synchronize()
        d_ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(5)]))
        d_bytes = 4 * wl.H_q * Ld + wl.H_q * kd * (2 * wl.d * 2 + 4)     # z once; K, V rows and z of the kept keys
        out["decode"] = {"workload": f"1 x {Ld}-token cache, H_q={wl.H_q} H_kv={wl.H_kv} d={wl.d} k={kd}", "ms": d_ms,
                         "algorithmic_bytes": d_bytes, "GB/s": d_bytes / (d_ms * 1e-3) / 1e9, "hbm_peak_GB/s": 8000.0}
        # the same cache in a decode loop: kept sets carried over and updated with the newest key only
        lens = torch.tensor([Ld - 8], dtype=torch.int32, device=dev)
        B.dma_decode_step(dshape, qc, Kc, Vc, zc, cuc, lens, True, oc, lc, kc, kb)
        st_ms = []
        for i in range(6):
            lens.add_(1)
            ev[0].record()
            B.dma_decode_step(dshape, qc, Kc, Vc, zc, cuc, lens, False, oc, lc, kc, kb)
            ev[1].record()
            torch.cuda.synchronize()
            st_ms.append(ev[0].elapsed_time(ev[1]))
        s_ms = float(np.median(st_ms[1:]))
        s_bytes = wl.H_q * kd * (2 * wl.d * 2 + 4 + 4 + 4)       # K, V rows, z (twice) and index of the kept keys
        out["decode_step"] = {"ms": s_ms, "algorithmic_bytes": s_bytes, "GB/s": s_bytes / (s_ms * 1e-3) / 1e9}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, wl, flops / wl.H_q)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
