"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle.

Index work (expiry, kept-key lists) must match bit for bit when both sides see
the same fp32 scores; floating-point outputs must meet the tolerances in
gpu_harness.tol().  The attention comparisons feed the oracle the scores the GPU
produced (widened exactly to fp64), so both sides select on identical keys; the
scores themselves are compared with the oracle's own Eq. 3 separately.
"""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2508_02124_amd import binding as B
from paper_2508_02124_amd import workloads as wlmod
from gpu_harness import (BF16_SUM_SREL, BQ, DEGENERATE_K, DeviceCase, check_close, degenerate_sum_allowance,
                         tol)

pytestmark = pytest.mark.gpu

SMALL = {
    "cfg1": lambda: wlmod.CONFIGS["cfg1"],
    "ragged_varlen_d64": lambda: wlmod.small_workload("ragged_varlen_d64", 11, 4, 2, 64, 48, (200, 77, 300, 1, 129)),
    "ragged_d128": lambda: wlmod.small_workload("ragged_d128", 12, 2, 1, 128, 100, (333,)),
    "k_ge_len": lambda: wlmod.small_workload("k_ge_len", 13, 4, 4, 64, 512, (150, 150)),
    "empty_doc": lambda: wlmod.small_workload("empty_doc", 14, 2, 2, 64, 32, (100, 0, 60)),
    "multi_tile_d128": lambda: wlmod.small_workload("multi_tile_d128", 15, 4, 2, 128, 160, (700, 260)),
    # degenerate shapes: one-token and few-token documents, k = 1, a single token in total, k = 2 across
    # several blocks (almost every key is evicted at once), 8 q-heads per kv-head, 3 q-heads (not a multiple of 8)
    "tiny_docs": lambda: wlmod.small_workload("tiny_docs", 16, 2, 2, 64, 2, (1, 2, 1, 3, 64, 65, 1)),
    "k1_d128": lambda: wlmod.small_workload("k1_d128", 17, 2, 1, 128, 1, (300,)),
    "single_token": lambda: wlmod.small_workload("single_token", 18, 2, 2, 64, 4, (1,)),
    "more_docs_than_tokens": lambda: wlmod.small_workload("more_docs_than_tokens", 25, 4, 2, 128, 256, (0, 1, 0)),
    "k2_many_blocks": lambda: wlmod.small_workload("k2_many_blocks", 19, 3, 3, 64, 2, (900,)),
    "gqa8_d64": lambda: wlmod.small_workload("gqa8_d64", 20, 8, 1, 64, 70, (520,)),
    # head dimension 256: ragged documents over several tiles, a window wider than a document, k = 2, GQA
    "ragged_d256": lambda: wlmod.small_workload("ragged_d256", 26, 4, 2, 256, 100, (333, 70, 0, 129)),
    "multi_tile_d256": lambda: wlmod.small_workload("multi_tile_d256", 27, 2, 1, 256, 160, (700, 260)),
    "k2_d256": lambda: wlmod.small_workload("k2_d256", 28, 2, 2, 256, 2, (530,)),
    "k_ge_len_d256": lambda: wlmod.small_workload("k_ge_len_d256", 29, 4, 1, 256, 512, (150, 290)),
    # 600 short documents (1..12 tokens, a few empty): block table, per-document sorts and plans at scale
    "many_tiny_docs": lambda: wlmod.small_workload(
        "many_tiny_docs", 24, 2, 1, 64, 5, tuple(int(x) for x in np.random.default_rng(24).integers(0, 13, 600))),
}


def tie_scores(H, T, seed, levels=6):
    r = np.random.default_rng(seed)
    return (r.integers(1, levels + 1, size=(H, T)) / levels).astype(np.float32)


def check_mask(case: DeviceCase, label):
    inp, wl = case.inp, case.wl
    cu = inp.cu_seqlens
    zg = case.host("z").astype(np.float64)
    eg = case.host("expiry")
    if not case.z_given:
        zo = orc.z_scores(inp.V, inp.W, inp.A, wl.H_q)
        rel = np.abs(zg - zo) / np.abs(zo)
        assert rel.max() <= 1e-5, f"{label}: z rel err {rel.max():.3e}"
    n_sel_diff = 0
    for h in range(wl.H_q):
        for a, b in zip(cu[:-1], cu[1:]):
            if b == a:
                continue
            e = orc.expiry_sequential(zg[h, a:b], wl.k) + a
            assert (eg[h, a:b] == e).all(), f"{label}: expiry mismatch head {h} doc [{a},{b})"
            if not case.z_given:
                n_sel_diff += int((orc.expiry_sequential(zo[h, a:b], wl.k) + a != e).sum())
    if case.topk is not None:
        tk = case.host("topk")
        for h in range(wl.H_q):
            for a, b in zip(cu[:-1], cu[1:]):
                if b == a:
                    continue
                ref = orc.topk_indices(zg[h, a:b], wl.k)
                ref = np.where(ref >= 0, ref + a, -1)
                assert (tk[h, a:b] == ref).all(), f"{label}: topk_idx mismatch head {h}"
    # plan structure: clean residents + partial list == keys active in the block
    pv = case.plan_views()
    assert pv["block_rows"] == BQ
    nblk = sum((int(b - a) + BQ - 1) // BQ for a, b in zip(cu[:-1], cu[1:]))
    assert pv["nblk"] == nblk
    bi = 0
    for d, (a, b) in enumerate(zip(cu[:-1], cu[1:])):
        for r0 in range(a, b, BQ):
            r1 = min(r0 + BQ, b)
            assert pv["blk"][bi].tolist() == [d, r0, r1, a]
            for h in range(wl.H_q):
                j = np.arange(a, r1)
                e = eg[h, a:r1]
                active = j[e > np.maximum(j, r0)]
                clean = j[(j < r0) & (e > r1 - 1)]
                row = pv["slot"][h, bi]
                got_clean = row[row >= 0]
                assert len(set(got_clean.tolist())) == got_clean.size
                assert sorted(got_clean.tolist()) == clean.tolist(), f"{label}: slot table block {bi} head {h}"
                assert (row[min(wl.k, r0 - a):] == -1).all()
                pc = pv["pcnt"][h, bi]
                part = pv["plist"][h, bi, :pc]
                assert len(set(part.tolist())) == pc
                assert sorted(part.tolist()) == sorted(set(active.tolist()) - set(clean.tolist())), \
                    f"{label}: partial list block {bi} head {h}"
            bi += 1
    return n_sel_diff


def test_plan_window_wider_than_one_column_tile(gpu):
    """k = 5000: the slot table is written in two column tiles (4096 + 1024 columns)."""
    print("[case] plan wide window", flush=True)
    wl = wlmod.small_workload("wide_window", 24, 2, 1, 64, 5000, (7000, 300, 5300))
    inp = wlmod.make_inputs(wl)
    case = DeviceCase(inp, gpu)
    case.mask_gen()
    print("  selection differences vs fp64 scores:", check_mask(case, "wide_window"), flush=True)


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_mask_gen_and_forward_small(gpu, name, dtype):
    run_mask_gen_and_forward(gpu, SMALL[name](), dtype)


def run_mask_gen_and_forward(gpu, wl, dtype):
    name = wl.name
    print(f"[case] mask+fwd {name} {dtype}", flush=True)
    inp = wlmod.make_inputs(wl, dtype=dtype)
    case = DeviceCase(inp, gpu, topk=True)
    case.mask_gen()
    nd = check_mask(case, f"{name}/{dtype}")
    print(f"  selection differences oracle-z vs gpu-z: {nd}", flush=True)
    case.fwd()
    zg = case.host("z").astype(np.float64)
    O, LSE = orc.dma_forward(inp.Q, inp.K, inp.V, zg, inp.cu_seqlens, inp.wl.k)
    t = tol(dtype == "bf16")
    print("  O", check_close("O", case.host("O"), O, **t), flush=True)
    print("  LSE", check_close("LSE", case.host("LSE"), LSE, **tol(False) if dtype == "f32" else
                               dict(atol=2e-2, rtol=1e-2, frob=1e-2)), flush=True)


@pytest.mark.parametrize("levels", [1, 6])
def test_mask_gen_heavy_ties_supplied_scores(gpu, levels):
    print(f"[case] ties levels={levels}", flush=True)
    wl = wlmod.small_workload("ties", 21, 4, 2, 64, 70, (500, 140))
    inp = wlmod.make_inputs(wl)
    z = tie_scores(wl.H_q, inp.T, 5, levels)
    case = DeviceCase(inp, gpu, z_override=z, topk=True)
    case.mask_gen()
    check_mask(case, f"ties{levels}")
    assert (case.host("z") == z).all()                   # supplied scores are left untouched
    case.fwd()
    O, LSE = orc.dma_forward(inp.Q, inp.K, inp.V, z.astype(np.float64), inp.cu_seqlens, wl.k)
    check_close("O", case.host("O"), O, **tol(True))
    check_close("LSE", case.host("LSE"), LSE, **tol(True))


def test_dense_equivalence_zero_scores(gpu):
    """k >= L and z = 0: the path must reduce to plain causal attention (torch SDPA in fp32 as a
    second, independent reference next to the oracle)."""
    print("[case] dense equivalence", flush=True)
    wl = wlmod.small_workload("dense", 22, 4, 2, 128, 400, (384,))
    inp = wlmod.make_inputs(wl)
    case = DeviceCase(inp, gpu, z_override=np.zeros((wl.H_q, inp.T), np.float32))
    case.mask_gen()
    case.fwd()
    q = torch.tensor(inp.Q).permute(1, 0, 2)[None]
    k = torch.tensor(inp.K).permute(1, 0, 2)[None].repeat_interleave(2, dim=1)
    v = torch.tensor(inp.V).permute(1, 0, 2)[None].repeat_interleave(2, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)[0].permute(1, 0, 2).numpy()
    check_close("O vs SDPA", case.host("O"), ref, **tol(True))
    O, _ = orc.dma_forward(inp.Q, inp.K, inp.V, np.zeros((wl.H_q, inp.T)), inp.cu_seqlens, wl.k)
    check_close("O vs oracle", case.host("O"), O, **tol(True))


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_backward_small(gpu, name, dtype):
    run_backward(gpu, SMALL[name](), dtype)


def check_gradients(case, zg, dtype, causal=True, label=""):
    """dQ, dK, dV, dz of the device case against the oracle at the plain tolerance.

    Alg. 2 loads O and the row statistics from memory: D_i = rowsum(dO_i o O_i) and P_ij = exp(S_ij - LSE_i)
    are formed from the buffers that dma_bwd was handed (bf16 O, fp32 LSE), so the oracle takes those same
    buffers (O_stored, LSE_stored) and the comparison measures the backward kernels' own rounding.  Only in
    the bf16 path, and only for keep windows of one to three keys, may a few dK / dV elements use the
    summand-mass allowance (see gpu_harness)."""
    inp, wl = case.inp, case.wl
    is_bf16 = dtype == "bf16"
    mass = {}
    dQ, dK, dV, dz = orc.dma_backward(inp.Q, inp.K, inp.V, zg, inp.dO, inp.cu_seqlens, wl.k, causal=causal,
                                      abs_out=mass, O_stored=case.host("O"), LSE_stored=case.host("LSE"))
    t = tol(is_bf16)
    print(f"  {label}dQ", check_close("dQ", case.host("dQ"), dQ, **t), flush=True)
    for nm, ref in (("dK", dK), ("dV", dV)):
        extra = {}
        if wl.k <= DEGENERATE_K and is_bf16:
            extra = dict(summand_abs=mass[nm], srel=BF16_SUM_SREL, max_beyond=degenerate_sum_allowance(ref))
        print(f"  {label}{nm}", check_close(nm, case.host(nm), ref, **extra, **t), flush=True)
    print(f"  {label}dz", check_close("dz", case.host("dz"), dz, **t), flush=True)
    # keys that are never kept get exactly zero gradient into z
    eg = case.host("expiry")
    never = eg == np.arange(inp.T)[None, :]
    assert (case.host("dz")[never] == 0.0).all()


def run_backward(gpu, wl, dtype):
    name = wl.name
    print(f"[case] bwd {name} {dtype}", flush=True)
    inp = wlmod.make_inputs(wl, dtype=dtype)
    case = DeviceCase(inp, gpu)
    case.mask_gen()
    case.fwd()
    case.bwd()
    zg = case.host("z").astype(np.float64)
    check_gradients(case, zg, dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_plan_decides_the_softmax_scale(gpu, dtype):
    """The plan holds z / scale and the scale itself; dma_fwd / dma_bwd take both from it, so a shape
    whose softmax_scale differs from the one given to dma_mask_gen cannot split the scores from their bias."""
    print(f"[case] plan-authoritative scale {dtype}", flush=True)
    wl = wlmod.small_workload("scale_in_plan", 31, 4, 2, 64 if dtype == "f32" else 128, 40, (300, 45))
    inp = wlmod.make_inputs(wl, dtype=dtype)
    case = DeviceCase(inp, gpu)
    case.shape.softmax_scale = 0.2
    case.mask_gen()
    case.shape.softmax_scale = 0.9            # not the plan's: must be ignored
    case.fwd()
    case.bwd()
    zg = case.host("z").astype(np.float64)
    t = tol(dtype == "bf16")
    O, LSE = orc.dma_forward(inp.Q, inp.K, inp.V, zg, inp.cu_seqlens, wl.k, scale=0.2)
    check_close("O", case.host("O"), O, **t)
    check_close("LSE", case.host("LSE"), LSE, **t)
    dQ, dK, dV, dz = orc.dma_backward(inp.Q, inp.K, inp.V, zg, inp.dO, inp.cu_seqlens, wl.k, scale=0.2,
                                      O_stored=case.host("O"), LSE_stored=case.host("LSE"))
    for nm, ref in (("dQ", dQ), ("dK", dK), ("dV", dV), ("dz", dz)):
        check_close(nm, case.host(nm), ref, **t)


@pytest.mark.parametrize("name", ["cfg1", "ragged_varlen_d64", "multi_tile_d128", "gqa8_d64", "many_tiny_docs"])
def test_backward_on_reference_forward_results(gpu, name):
    """dma_bwd as an entry point of its own: O and LSE are inputs.  It is handed the oracle's forward
    results (O rounded to bf16 on the host, LSE to fp32), the oracle forms D_i from that same O, and
    no device output other than the scores enters the reference."""
    wl = SMALL[name]()
    print(f"[case] bwd on reference O / LSE {wl.name}", flush=True)
    inp = wlmod.make_inputs(wl, dtype="bf16")
    case = DeviceCase(inp, gpu)
    case.mask_gen()
    zg = case.host("z").astype(np.float64)
    O, LSE = orc.dma_forward(inp.Q, inp.K, inp.V, zg, inp.cu_seqlens, wl.k)
    case.set_forward_results(O, LSE)
    case.bwd()
    check_gradients(case, zg, "bf16", label="(reference O) ")


def random_small_workloads(seed, count, head_dim=None):
    """Seeded random shapes around the tile edges (rows 31 ... 1100 per document, windows 1 ... 2000,
    1 - 6 documents including empty ones, G = 1, 2, 4, head dimension 64 or 128 -- or head_dim for
    all of them --, causal or not)."""
    import random
    rnd = random.Random(seed)
    out = []
    for it in range(count):
        d = rnd.choice([64, 128])
        d = d if head_dim is None else head_dim
        H_kv = rnd.choice([1, 2, 3])
        G = rnd.choice([1, 2, 4])
        ndocs = rnd.choice([1, 1, 2, 3, 6])
        seqlens = tuple(rnd.choice([0, 1, 2, 31, 64, 100, 255, 256, 257, 300, 511, 700, 1100]) for _ in range(ndocs))
        if sum(seqlens) == 0:
            seqlens = seqlens + (130,)
        k = rnd.choice([1, 2, 3, 17, 64, 100, 128, 129, 256, 300, 640, 2000])
        causal = rnd.random() < 0.75
        dtype = rnd.choice(["bf16", "f32"])
        out.append((wlmod.small_workload(f"rnd{seed}_{it}", 5000 + 100 * seed + it, H_kv * G, H_kv, d, k, seqlens,
                                         causal=causal), dtype))
    return out


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_small_shapes(gpu, seed):
    for wl, dtype in random_small_workloads(seed, 14):
        print(f"[shape] H_q={wl.H_q} H_kv={wl.H_kv} d={wl.d} k={wl.k} seqlens={wl.seqlens} causal={wl.causal}", flush=True)
        if wl.causal:
            run_mask_gen_and_forward(gpu, wl, dtype)
            run_backward(gpu, wl, dtype)
        else:
            run_noncausal(gpu, wl, dtype)


def test_random_small_shapes_head_dim_256(gpu):
    for wl, dtype in random_small_workloads(4, 12, head_dim=256):
        print(f"[shape] H_q={wl.H_q} H_kv={wl.H_kv} d={wl.d} k={wl.k} seqlens={wl.seqlens} causal={wl.causal}", flush=True)
        if wl.causal:
            run_mask_gen_and_forward(gpu, wl, dtype)
            run_backward(gpu, wl, dtype)
        else:
            run_noncausal(gpu, wl, dtype)


def test_backward_heavy_ties(gpu):
    print("[case] bwd ties", flush=True)
    wl = wlmod.small_workload("ties", 21, 4, 2, 128, 70, (500, 140))
    inp = wlmod.make_inputs(wl)
    z = tie_scores(wl.H_q, inp.T, 6, 4)
    case = DeviceCase(inp, gpu, z_override=z)
    case.mask_gen()
    case.fwd()
    case.bwd()
    check_gradients(case, z.astype(np.float64), "bf16")


# ----------------------------------------------------------------------------- gradient of the content scores
MASK_BWD_CASES = {
    # name: (T, H_q, H_kv, d)  -- several 64-token tiles with a ragged tail, G = 1, 2, 4, 8, 16
    "tail_d64": (333, 4, 2, 64),
    "g1_d128": (200, 3, 3, 128),
    "g8_d128": (1000, 8, 1, 128),
    "tiny": (5, 2, 1, 64),
    "g16_d64": (300, 16, 1, 64),          # more than 8 q-heads per kv-head: the LDS-based kernel
    "many_tiles_d128": (70000, 4, 1, 128),  # several tiles per workgroup
    "tail_d256": (333, 4, 2, 256),          # 32-token tiles at 256 channels
    "many_tiles_d256": (40000, 8, 1, 256),
}


@pytest.mark.parametrize("name", list(MASK_BWD_CASES))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_mask_backward(gpu, name, dtype):
    print(f"[case] mask_bwd {name} {dtype}", flush=True)
    import torch
    T, H_q, H_kv, d = MASK_BWD_CASES[name]
    r = np.random.default_rng(100 + list(MASK_BWD_CASES).index(name))
    V = r.standard_normal((T, H_kv, d)).astype(np.float32)
    if dtype == "bf16":
        V = wlmod.bf16_bits_to_f32(wlmod.f32_to_bf16_bits(V))
    W = (r.standard_normal((H_q, d)) / np.sqrt(d)).astype(np.float32)
    A = (-r.uniform(0.5, 2.0, H_q)).astype(np.float32)
    dz = r.standard_normal((H_q, T)).astype(np.float32)
    dV0 = r.standard_normal((T, H_kv, d)).astype(np.float32)
    if dtype == "bf16":
        dV0 = wlmod.bf16_bits_to_f32(wlmod.f32_to_bf16_bits(dV0))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    shape = B.make_shape(T=T, n_docs=1, H_q=H_q, H_kv=H_kv, d=d, k=1,
                         dtype=B.DMA_BF16 if dtype == "bf16" else B.DMA_F32)
    dev = lambda x, dt=None: torch.from_numpy(np.ascontiguousarray(x)).to(gpu).to(dt or torch.float32)
    Vd, Wd, Ad, dzd = dev(V, tdt), dev(W), dev(A), dev(dz)
    dWd = torch.full((H_q, d), 7.0, device=gpu)          # outputs are overwritten, whatever they held
    dAd = torch.full((H_q,), -3.0, device=gpu)
    dVd = torch.full((T, H_kv, d), 5.0, device=gpu, dtype=tdt)
    B.dma_mask_bwd(shape, Vd, Wd, Ad, dzd, dWd, dAd, dVd, False)
    dW, dA, dVz = orc.mask_backward(V, W, A, dz, H_q)
    t = tol(dtype == "bf16")
    t32 = dict(atol=1e-4, rtol=1e-4, frob=1e-5)           # fp32 sums over T rows, fp32 exp / log
    print("  dW", check_close("dW", dWd.cpu().numpy(), dW, **t32), flush=True)
    print("  dA", check_close("dA", dAd.cpu().numpy(), dA, **t32), flush=True)
    print("  dVz", check_close("dVz", dVd.float().cpu().numpy(), dVz, **(t if dtype == "bf16" else t32)), flush=True)
    # accumulate into an existing dV
    dVd2 = dev(dV0, tdt)
    B.dma_mask_bwd(shape, Vd, Wd, Ad, dzd, dWd, dAd, dVd2, True)
    print("  dV+=", check_close("dV+dVz", dVd2.float().cpu().numpy(), dV0 + dVz, **(t if dtype == "bf16" else t32)), flush=True)
    print("  dW again", check_close("dW", dWd.cpu().numpy(), dW, **t32), flush=True)


# ----------------------------------------------------------------------------- without the causal restriction
NONCAUSAL = {
    "nc_ragged_varlen_d64": lambda: wlmod.small_workload("nc_ragged_varlen_d64", 41, 4, 2, 64, 48, (200, 77, 300, 1, 129), causal=False),
    "nc_multi_tile_d128": lambda: wlmod.small_workload("nc_multi_tile_d128", 42, 4, 2, 128, 160, (700, 260), causal=False),
    "nc_k_ge_len": lambda: wlmod.small_workload("nc_k_ge_len", 43, 4, 4, 64, 512, (150, 0, 150), causal=False),
    "nc_more_docs_than_tokens": lambda: wlmod.small_workload("nc_more_docs_than_tokens", 47, 4, 2, 128, 256, (0, 1), causal=False),
    "nc_k1_d128": lambda: wlmod.small_workload("nc_k1_d128", 44, 2, 1, 128, 1, (300,), causal=False),
    "nc_k_not_tile_multiple": lambda: wlmod.small_workload("nc_k_not_tile_multiple", 45, 3, 3, 64, 130, (1000,), causal=False),
}


def check_noncausal_mask(case, label):
    """expiry = end of the document for the document's min(k, n) best keys, own index otherwise;
    topk_idx: that set on every row; plan: every block of the document lists exactly that set, no
    partial keys."""
    inp, wl = case.inp, case.wl
    cu = inp.cu_seqlens
    zg = case.host("z").astype(np.float64)
    eg = case.host("expiry")
    tk = case.host("topk")
    pv = case.plan_views()
    bi = 0
    for d, (a, b) in enumerate(zip(cu[:-1], cu[1:])):
        n = int(b - a)
        if n == 0:
            continue
        nb = (n + BQ - 1) // BQ
        for h in range(wl.H_q):
            kept = orc.kept_mask_definition(zg[h, a:b], wl.k, causal=False)
            assert (kept == kept[0]).all()
            ref_e = np.where(kept[0], b, np.arange(a, b))
            assert (eg[h, a:b] == ref_e).all(), f"{label}: expiry head {h} doc {d}"
            ref_tk = orc.topk_indices(zg[h, a:b], wl.k, causal=False)
            assert (tk[h, a:b] == np.where(ref_tk >= 0, ref_tk + a, -1)).all(), f"{label}: topk_idx head {h} doc {d}"
            want = (np.flatnonzero(kept[0]) + a).tolist()
            for blk in range(bi, bi + nb):
                row = pv["slot"][h, blk]
                assert sorted(row[row >= 0].tolist()) == want, f"{label}: slot table block {blk} head {h}"
                assert (row[min(wl.k, n):] == -1).all()
                assert pv["pcnt"][h, blk] == 0
        bi += nb
    assert pv["nblk"] == bi


@pytest.mark.parametrize("name", list(NONCAUSAL))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_noncausal_small(gpu, name, dtype):
    run_noncausal(gpu, NONCAUSAL[name](), dtype)


def run_noncausal(gpu, wl, dtype):
    name = wl.name
    print(f"[case] non-causal {name} {dtype}", flush=True)
    inp = wlmod.make_inputs(wl, dtype=dtype)
    case = DeviceCase(inp, gpu, topk=True)
    case.mask_gen()
    check_noncausal_mask(case, f"{name}/{dtype}")
    case.fwd()
    case.bwd()
    zg = case.host("z").astype(np.float64)
    O, LSE = orc.dma_forward(inp.Q, inp.K, inp.V, zg, inp.cu_seqlens, wl.k, causal=False)
    t = tol(dtype == "bf16")
    print("  O", check_close("O", case.host("O"), O, **t), flush=True)
    print("  LSE", check_close("LSE", case.host("LSE"), LSE, **t), flush=True)
    check_gradients(case, zg, dtype, causal=False)


def test_noncausal_ties_supplied_scores(gpu):
    print("[case] non-causal ties", flush=True)
    wl = wlmod.small_workload("nc_ties", 46, 4, 2, 64, 70, (500, 140), causal=False)
    inp = wlmod.make_inputs(wl)
    z = tie_scores(wl.H_q, inp.T, 9, 4)
    case = DeviceCase(inp, gpu, z_override=z, topk=True)
    case.mask_gen()
    check_noncausal_mask(case, "nc_ties")
    case.fwd()
    O, LSE = orc.dma_forward(inp.Q, inp.K, inp.V, z.astype(np.float64), inp.cu_seqlens, wl.k, causal=False)
    check_close("O", case.host("O"), O, **tol(True))
    check_close("LSE", case.host("LSE"), LSE, **tol(True))


# ----------------------------------------------------------------------------- cross-head scores (Eq. 3, full Delta)
XHEAD_CASES = {
    # name: (T, H_q, H_kv, d)
    "ragged_d64": (517, 6, 3, 64),
    "bench_heads_d128": (300, 32, 8, 128),
    "one_tile_d128": (64, 2, 1, 128),
    "odd_heads_d64": (1000, 5, 1, 64),
    "many_tiles_d128": (40000, 12, 4, 128),      # several tiles per workgroup in the backward
}


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("name", list(XHEAD_CASES))
def test_xhead_scores_and_backward(gpu, name, dtype):
    print(f"[case] xhead {name} {dtype}", flush=True)
    import torch
    T, H_q, H_kv, d = XHEAD_CASES[name]
    r = np.random.default_rng(200 + list(XHEAD_CASES).index(name))
    V = r.standard_normal((T, H_kv, d)).astype(np.float32)
    dV0 = r.standard_normal((T, H_kv, d)).astype(np.float32)
    if dtype == "bf16":
        V = wlmod.bf16_bits_to_f32(wlmod.f32_to_bf16_bits(V))
        dV0 = wlmod.bf16_bits_to_f32(wlmod.f32_to_bf16_bits(dV0))
    Delta = (r.standard_normal((H_q, H_kv * d)) / np.sqrt(H_kv * d)).astype(np.float32)
    A = (-r.uniform(0.5, 2.0, H_q)).astype(np.float32)
    dz = r.standard_normal((H_q, T)).astype(np.float32)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    shape = B.make_shape(T=T, n_docs=1, H_q=H_q, H_kv=H_kv, d=d, k=1,
                         dtype=B.DMA_BF16 if dtype == "bf16" else B.DMA_F32)
    dev = lambda x, dt=None: torch.from_numpy(np.ascontiguousarray(x)).to(gpu).to(dt or torch.float32)
    Vd, Dd, Ad, dzd = dev(V, tdt), dev(Delta), dev(A), dev(dz)
    zd = torch.full((H_q, T), float("nan"), device=gpu)
    B.dma_scores_xhead(shape, Vd, Dd, Ad, zd)
    zr = orc.z_scores_xhead(V, Delta, A)
    zg = zd.cpu().numpy().astype(np.float64)
    assert np.isfinite(zg).all()
    rel = np.abs(zg - zr) / zr
    print("  z max rel", rel.max(), flush=True)
    assert rel.max() <= 1e-5
    dDd = torch.full((H_q, H_kv * d), 7.0, device=gpu)       # outputs are overwritten, whatever they held
    dAd = torch.full((H_q,), -3.0, device=gpu)
    dVd = torch.full((T, H_kv, d), 5.0, device=gpu, dtype=tdt)
    B.dma_scores_xhead_bwd(shape, Vd, Dd, Ad, dzd, dDd, dAd, dVd, False)
    dD, dA, dVz = orc.xhead_backward(V, Delta, A, dz)
    t = tol(dtype == "bf16")
    t32 = dict(atol=1e-4, rtol=1e-4, frob=1e-5)               # fp32 sums over T rows, fp32 exp / log
    if T > 10000:
        t32 = dict(atol=1e-3, rtol=1e-4, frob=1e-5)           # sums of 40000 terms of order one
    print("  dDelta", check_close("dDelta", dDd.cpu().numpy(), dD, **t32), flush=True)
    print("  dA", check_close("dA", dAd.cpu().numpy(), dA, **t32), flush=True)
    tv = t if dtype == "bf16" else dict(atol=1e-4, rtol=1e-4, frob=1e-5)
    print("  dVz", check_close("dVz", dVd.float().cpu().numpy(), dVz, **tv), flush=True)
    dVd2 = dev(dV0, tdt)
    B.dma_scores_xhead_bwd(shape, Vd, Dd, Ad, dzd, dDd, dAd, dVd2, True)
    print("  dV+=", check_close("dV+dVz", dVd2.float().cpu().numpy(), dV0 + dVz, **tv), flush=True)
    print("  dDelta again", check_close("dDelta", dDd.cpu().numpy(), dD, **t32), flush=True)


@pytest.mark.gpu
def test_xhead_block_structure_equals_per_head_path(gpu):
    """A Delta that is zero outside the block of each head's own kv-head gives the scores of the
    per-head entry point (dma_mask_gen with W), to fp32 rounding."""
    print("[case] xhead vs per-head", flush=True)
    import torch
    wl = wlmod.small_workload("xh", 23, 8, 2, 128, 50, (700,))
    inp = wlmod.make_inputs(wl)
    case = DeviceCase(inp, gpu)
    case.mask_gen()
    G = wl.H_q // wl.H_kv
    Delta = np.zeros((wl.H_q, wl.H_kv * wl.d), dtype=np.float32)
    for h in range(wl.H_q):
        Delta[h, (h // G) * wl.d:(h // G + 1) * wl.d] = inp.W[h]
    z2 = torch.empty_like(case.z)
    B.dma_scores_xhead(case.shape, case.V, torch.from_numpy(Delta).to(gpu), case.A, z2)
    a, b = case.host("z").astype(np.float64), z2.cpu().numpy().astype(np.float64)
    assert (np.abs(a - b) / a).max() <= 2e-6


# ----------------------------------------------------------------------------- decode (newest row of every sequence)
DECODE_CASES = {
    # name: (doc lengths, H_q, H_kv, d, k, tie levels or 0)
    "varlen_d64": ((300, 0, 1, 70, 1500), 4, 2, 64, 64, 0),
    "gqa_d128": ((2500, 129), 8, 2, 128, 128, 0),
    "ties": ((900, 400), 2, 2, 64, 100, 5),
    "k_ge_len": ((50, 200), 2, 1, 128, 512, 0),
    "gqa_d256": ((1300, 0, 257), 4, 2, 256, 96, 0),
}


@pytest.mark.parametrize("name", list(DECODE_CASES))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_decode(gpu, name, dtype):
    print(f"[case] decode {name} {dtype}", flush=True)
    lens, H_q, H_kv, d, k, levels = DECODE_CASES[name]
    r = np.random.default_rng(200 + list(DECODE_CASES).index(name))
    T, n_docs = sum(lens), len(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rnd = lambda *s: r.standard_normal(s).astype(np.float32)
    q, K, V = rnd(n_docs, H_q, d), rnd(T, H_kv, d), rnd(T, H_kv, d)
    z = r.uniform(0.05, 1.0, size=(H_q, T)).astype(np.float32)
    if levels:
        z = (np.round(z * levels) / levels + 0.125).astype(np.float32)     # heavy ties across the threshold
    if dtype == "bf16":
        q, K, V = (wlmod.bf16_bits_to_f32(wlmod.f32_to_bf16_bits(x)) for x in (q, K, V))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    shape = B.make_shape(T=T, n_docs=n_docs, H_q=H_q, H_kv=H_kv, d=d, k=k,
                         dtype=B.DMA_BF16 if dtype == "bf16" else B.DMA_F32)
    dev = lambda x, dt=torch.float32: torch.from_numpy(np.ascontiguousarray(x)).to(gpu).to(dt)
    kcap = min(k, T)
    kept = torch.full((n_docs, H_q, kcap), -7, dtype=torch.int32, device=gpu)
    o = torch.full((n_docs, H_q, d), 3.0, dtype=tdt, device=gpu)
    lse = torch.full((H_q, n_docs), 3.0, device=gpu)
    nb = B.dma_decode_kept_bytes(shape)
    assert nb >= kept.numel() * 4
    pad = torch.empty(nb, dtype=torch.uint8, device=gpu)                  # buffer of exactly the requested size
    kept_buf = pad[:kept.numel() * 4].view(torch.int32).view(n_docs, H_q, kcap)
    B.dma_decode(shape, dev(q, tdt), dev(K, tdt), dev(V, tdt), dev(z), torch.from_numpy(cu).to(gpu), o, lse,
                 kept_buf, nb)
    ro, rl, rk = orc.dma_decode(q, K, V, z, cu, k)
    got_k = kept_buf.cpu().numpy()
    for b in range(n_docs):
        kk = rk[b].shape[1]
        assert (got_k[b, :, :kk] == rk[b]).all(), f"kept set of sequence {b}"     # bit-exact, ascending
    t = tol(dtype == "bf16")
    print("  o", check_close("o", o.float().cpu().numpy(), ro, **t), flush=True)
    got_l = lse.cpu().numpy()
    fin = np.isfinite(rl)
    assert (np.isneginf(got_l) == ~fin).all()
    print("  lse", check_close("lse", got_l[fin], rl[fin], **(t if dtype == "bf16" else tol(False))), flush=True)
    with pytest.raises(B.DmaError) as e:                                    # kept buffer too small
        B.dma_decode(shape, dev(q, tdt), dev(K, tdt), dev(V, tdt), dev(z), torch.from_numpy(cu).to(gpu), o, lse,
                     kept_buf, nb - 256 if nb > 256 else 0)
    assert e.value.status == B.DMA_EWORKSPACE


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_decode_step_loop(gpu, dtype):
    """A decode loop over sequences in fixed-capacity regions: the first call selects the kept sets,
    every later call updates them with the newest key only.  After every step the kept sets must be
    exactly the oracle's top-k of the current prefix (one sequence crosses from "fewer than k keys" to
    "full", one starts empty, one head has heavy ties), and o / lse must match."""
    print(f"[case] decode step loop {dtype}", flush=True)
    caps, lens0, steps = (400, 64, 900), (120, 0, 700), 45
    H_q, H_kv, d, k = 4, 2, 64, 130
    T = sum(caps)
    starts = np.concatenate([[0], np.cumsum(caps)]).astype(np.int32)
    r = np.random.default_rng(61)
    rnd = lambda shape: r.standard_normal(shape).astype(np.float32)
    K, V = rnd((T, H_kv, d)), rnd((T, H_kv, d))
    if dtype == "bf16":
        K, V = (wlmod.bf16_bits_to_f32(wlmod.f32_to_bf16_bits(x)) for x in (K, V))
    z = r.uniform(0.05, 1.0, size=(H_q, T)).astype(np.float32)
    z[2] = np.round(z[2] * 8) / 8                         # heavy ties
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x)).to(gpu).to(dt)
    Kd, Vd, zd, cud = dev(K, tdt), dev(V, tdt), dev(z, torch.float32), dev(starts, torch.int32)
    shape = B.make_shape(T=T, n_docs=len(caps), H_q=H_q, H_kv=H_kv, d=d, k=k,
                         dtype=B.DMA_BF16 if dtype == "bf16" else B.DMA_F32)
    kb = B.dma_decode_kept_bytes(shape)
    kept = torch.full((kb // 4,), -5, dtype=torch.int32, device=gpu)
    o = torch.empty((len(caps), H_q, d), dtype=tdt, device=gpu)
    lse = torch.empty((H_q, len(caps)), device=gpu)
    t = tol(dtype == "bf16")
    for step in range(steps):
        lens = np.array([l0 + step for l0 in lens0], dtype=np.int32)
        q = rnd((len(caps), H_q, d))
        if dtype == "bf16":
            q = wlmod.bf16_bits_to_f32(wlmod.f32_to_bf16_bits(q))
        B.dma_decode_step(shape, dev(q, tdt), Kd, Vd, zd, cud, dev(lens, torch.int32), step == 0, o, lse, kept, kb)
        # the oracle sees the current contents packed
        rows = np.concatenate([np.arange(starts[b], starts[b] + lens[b]) for b in range(len(caps))]).astype(np.int64)
        cu_p = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        ro, rl, rk = orc.dma_decode(q, K[rows], V[rows], z[:, rows].astype(np.float64), cu_p, k)
        got_k = kept.cpu().numpy()[: len(caps) * H_q * k].reshape(len(caps), H_q, k)
        for b in range(len(caps)):
            kk = min(k, int(lens[b]))
            want = rk[b] - cu_p[b] + starts[b]            # [H_q, kk], packed row -> row of the capacity layout
            assert want.shape == (H_q, kk) and (got_k[b, :, :kk] == want).all(), f"step {step} sequence {b}: kept set"
        check_close(f"o step {step}", o.float().cpu().numpy(), ro, **t)
        gl = lse.cpu().numpy()
        empty = lens == 0                                  # an empty sequence: o = 0, lse = -inf on both sides
        assert (gl[:, empty] == -np.inf).all() and (rl[:, empty] == -np.inf).all()
        check_close(f"lse step {step}", gl[:, ~empty], rl[:, ~empty], **t)
    print("  all steps match", flush=True)
