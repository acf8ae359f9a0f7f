"""HIP graph capture of the entry points: nothing in them allocates, synchronises or records a memset,
so a caller may capture a step (or a decode step) once and replay it.  Every replay is checked against
the eager result, with eager work and synchronisation between the replays."""
import numpy as np
import pytest
import torch

from paper_2508_02124_amd import binding as B
from paper_2508_02124_amd import workloads as wlmod
from gpu_harness import DeviceCase, check_close, tol

pytestmark = pytest.mark.gpu


def test_training_step_replays_match_eager(gpu):
    print("[case] graph: mask_gen + fwd + bwd", flush=True)
    wl = wlmod.small_workload("graph", 51, 4, 2, 128, 96, (700, 300))
    inp = wlmod.make_inputs(wl)
    case = DeviceCase(inp, gpu)
    case.mask_gen(); case.fwd(); case.bwd()
    eager = {n: case.host(n).copy() for n in ("z", "expiry", "O", "LSE", "dQ", "dK", "dV", "dz")}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream, as torch asks
        case.mask_gen(); case.fwd(); case.bwd()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        case.mask_gen(); case.fwd(); case.bwd()
    t = tol(True)
    for rep in range(3):
        for name in ("O", "dQ", "dK", "dV", "dz", "LSE"):   # poison the outputs, then some eager work
            getattr(case, name).fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert (case.host("expiry") == eager["expiry"]).all() and (case.host("z") == eager["z"]).all()
        assert (case.host("O") == eager["O"]).all() and (case.host("LSE") == eager["LSE"]).all()
        assert (case.host("dQ") == eager["dQ"]).all()
        for name in ("dK", "dV", "dz"):                 # accumulated with atomics: last bits may differ
            check_close(f"{name} replay {rep}", case.host(name), eager[name], **t)
        case.fwd()                                      # eager work between the replays
        torch.cuda.synchronize()
    print("  three replays match", flush=True)


def test_decode_step_replays_match_eager(gpu):
    print("[case] graph: decode step", flush=True)
    cap, H_q, H_kv, d, k = 3000, 4, 2, 64, 128
    r = np.random.default_rng(52)
    dev = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x)).to(gpu).to(dt)
    K = dev(r.standard_normal((cap, H_kv, d)).astype(np.float32), torch.bfloat16)
    V = dev(r.standard_normal((cap, H_kv, d)).astype(np.float32), torch.bfloat16)
    z = dev(r.uniform(0.05, 1.0, (H_q, cap)).astype(np.float32), torch.float32)
    q = dev(r.standard_normal((1, H_q, d)).astype(np.float32), torch.bfloat16)
    cu = torch.tensor([0, cap], dtype=torch.int32, device=gpu)
    shape = B.make_shape(T=cap, n_docs=1, H_q=H_q, H_kv=H_kv, d=d, k=k)
    kb = B.dma_decode_kept_bytes(shape)

    def run(n_steps, use_graph):
        kept = torch.zeros(kb // 4, dtype=torch.int32, device=gpu)
        o = torch.empty((1, H_q, d), dtype=torch.bfloat16, device=gpu)
        lse = torch.empty((H_q, 1), device=gpu)
        lens = torch.tensor([2000], dtype=torch.int32, device=gpu)
        B.dma_decode_step(shape, q, K, V, z, cu, lens, True, o, lse, kept, kb)
        torch.cuda.synchronize()
        graph = None
        if use_graph:
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):   # one step: the length grows on the device, then the call
                lens.add_(1)
                B.dma_decode_step(shape, q, K, V, z, cu, lens, False, o, lse, kept, kb)
        outs = []
        for _ in range(n_steps):
            if use_graph:
                graph.replay()
            else:
                lens.add_(1)
                B.dma_decode_step(shape, q, K, V, z, cu, lens, False, o, lse, kept, kb)
            torch.cuda.synchronize()
            outs.append((o.float().cpu().numpy().copy(), lse.cpu().numpy().copy(), kept[: H_q * k].cpu().numpy().copy()))
        return outs

    eager = run(6, False)
    replayed = run(6, True)      # (capture does not execute: the first replay is step 1)
    for s, (a, b) in enumerate(zip(eager, replayed)):
        assert (a[2] == b[2]).all(), f"kept sets differ at step {s}"
        assert (a[0] == b[0]).all() and (a[1] == b[1]).all(), f"outputs differ at step {s}"
    print("  six replayed steps match the eager loop", flush=True)
