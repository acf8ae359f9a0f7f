"""GPU parity of the caller-supplied attention bias (one value per key, with head and batch
broadcasting; Section 1 "Kernel Design"): dma_mask_gen_bias + dma_fwd + dma_bwd + dma_bias_bwd through
the C ABI against the oracle.  The bias must not move the kept sets (selection ranks z alone)."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2508_02124_amd import binding as B
from paper_2508_02124_amd import torch_api
from paper_2508_02124_amd import workloads as wlmod
from gpu_harness import DeviceCase, check_close, to_dev, tol

pytestmark = pytest.mark.gpu

FORMS = {  # name: (bias_heads as "all" / 1, per_token)
    "per_head_per_token": ("all", True),
    "head_broadcast": (1, True),
    "batch_broadcast": ("all", False),
    "head_and_batch_broadcast": (1, False),
}


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("form", list(FORMS))
def test_bias_forward_backward(gpu, form, dtype):
    print(f"[case] attention bias {form} {dtype}", flush=True)
    wl = wlmod.small_workload(f"bias_{form}", 71, 4, 2, 128 if dtype == "bf16" else 64, 40, (300, 77, 0, 260))
    inp = wlmod.make_inputs(wl, dtype=dtype)
    Hb = wl.H_q if FORMS[form][0] == "all" else 1
    per_token = FORMS[form][1]
    r = np.random.default_rng(72)
    n_cols = inp.T if per_token else inp.max_seqlen
    braw = (0.5 * r.standard_normal((Hb, n_cols))).astype(np.float32)   # (moderate: a peaked softmax is the k <= 3 regime)
    braw[:, 5] = -30.0                                    # a key masked for everyone (a large negative bias)
    case = DeviceCase(inp, gpu)
    bias_d = to_dev(braw, gpu)
    # the plain call first: the bias must not change scores or kept sets
    case.mask_gen()
    z0, e0 = case.host("z").copy(), case.host("expiry").copy()
    B.dma_mask_gen_bias(case.shape, case.V, case.W, case.A, case.cu, bias_d, Hb, per_token, case.z, case.expiry,
                        None, case.mask)
    assert np.array_equal(case.host("z"), z0) and np.array_equal(case.host("expiry"), e0)
    case.fwd()
    case.bwd()
    zg = z0.astype(np.float64)
    bias = orc.expand_bias(braw, wl.H_q, inp.cu_seqlens, per_token)
    O, LSE = orc.dma_forward(inp.Q, inp.K, inp.V, zg, inp.cu_seqlens, wl.k, bias=bias)
    t = tol(dtype == "bf16")
    print("  O", check_close("O", case.host("O"), O, **t), flush=True)
    print("  LSE", check_close("LSE", case.host("LSE"), LSE, **t), flush=True)
    dQ, dK, dV, dz = orc.dma_backward(inp.Q, inp.K, inp.V, zg, inp.dO, inp.cu_seqlens, wl.k, bias=bias,
                                      O_stored=case.host("O"), LSE_stored=case.host("LSE"))
    for nm, ref in (("dQ", dQ), ("dK", dK), ("dV", dV), ("dz", dz)):
        print(f"  {nm}", check_close(nm, case.host(nm), ref, **t), flush=True)
    dbias = torch.full((Hb, n_cols), float("nan"), device=gpu)
    B.dma_bias_bwd(case.shape, case.dz, case.cu, Hb, per_token, dbias)
    ref_db = orc.bias_backward(dz, Hb, inp.cu_seqlens, per_token, n_max=inp.max_seqlen)
    print("  dbias", check_close("dbias", dbias.cpu().numpy(), ref_db, **t), flush=True)
    # the masked key carries no weight: rows that keep it ignore it (its dz is ~0)
    assert np.abs(case.host("dz")[:, 5]).max() < 1e-6


def test_bias_argument_checks():
    from paper_2508_02124_amd import binding
    ok = B.make_shape(T=256, n_docs=2, H_q=4, H_kv=2, d=64, k=16, max_seqlen=200)
    p = 0x1000
    with pytest.raises(B.DmaError) as e:
        B.dma_mask_gen_bias(ok, p, p, p, p, None, 4, 1, p, p, None, p, stream=0)      # bias missing
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_mask_gen_bias(ok, p, p, p, p, p, 3, 1, p, p, None, p, stream=0)         # neither 1 nor H_q rows
    assert e.value.status == B.DMA_EINVAL
    nomax = B.make_shape(T=256, n_docs=2, H_q=4, H_kv=2, d=64, k=16)
    with pytest.raises(B.DmaError) as e:
        B.dma_mask_gen_bias(nomax, p, p, p, p, p, 1, 0, p, p, None, p, stream=0)      # shared row without max_seqlen
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_bias_bwd(ok, None, p, 1, 1, p, stream=0)                                 # dz missing
    assert e.value.status == B.DMA_EINVAL
    assert binding.dma_version() >= 130


def test_bias_through_autograd(gpu):
    print("[case] attention bias through the autograd function", flush=True)
    wl = wlmod.small_workload("bias_auto", 73, 4, 2, 64, 30, (150, 90))
    inp = wlmod.make_inputs(wl, dtype="f32")
    dev = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x)).to(gpu).to(dt)
    Q, K, V = (dev(getattr(inp, n), torch.float32).requires_grad_() for n in "QKV")
    W, A = dev(inp.W, torch.float32).requires_grad_(), dev(inp.A, torch.float32).requires_grad_()
    cu = dev(inp.cu_seqlens.astype(np.int32), torch.int32)
    braw = np.random.default_rng(74).standard_normal((1, inp.max_seqlen)).astype(np.float32)
    bias = dev(braw, torch.float32).requires_grad_()
    O = torch_api.dynamic_mask_attention(Q, K, V, W, A, cu, wl.k, inp.max_seqlen, 0.0, bias)
    O.backward(dev(inp.dO, torch.float32))
    torch.cuda.synchronize()
    zo = orc.z_scores(inp.V, inp.W, inp.A, wl.H_q)
    b = orc.expand_bias(braw, wl.H_q, inp.cu_seqlens, per_token=False)
    rO, _ = orc.dma_forward(inp.Q, inp.K, inp.V, zo, inp.cu_seqlens, wl.k, bias=b)
    _, _, _, rdz = orc.dma_backward(inp.Q, inp.K, inp.V, zo, inp.dO, inp.cu_seqlens, wl.k, bias=b)
    rdb = orc.bias_backward(rdz, 1, inp.cu_seqlens, per_token=False, n_max=inp.max_seqlen)
    t32 = dict(atol=1e-4, rtol=1e-4, frob=1e-4)      # (selection on the device's fp32 scores: no near-ties at this size)
    print("  O", check_close("O", O.detach().cpu().numpy(), rO, **t32), flush=True)
    print("  dbias", check_close("dbias", bias.grad.cpu().numpy(), rdb, **t32), flush=True)


def test_bias_at_the_cfg2_shape_dense(gpu):
    """The batch- and head-broadcast form (one bias row indexed by the position in the document) at
    2 x 4096 tokens, 16 / 4 heads, k = 1024: forward and backward dense against the oracle, and the
    bias gradient reduced over all heads and both documents."""
    print("[case] attention bias, head and batch broadcast, cfg2 shape dense", flush=True)
    inp = wlmod.make_inputs(wlmod.CONFIGS["cfg2"])
    wl = inp.wl
    braw = (0.5 * np.random.default_rng(73).standard_normal((1, inp.max_seqlen))).astype(np.float32)
    case = DeviceCase(inp, gpu)
    B.dma_mask_gen_bias(case.shape, case.V, case.W, case.A, case.cu, to_dev(braw, gpu), 1, False, case.z, case.expiry,
                        None, case.mask)
    case.fwd()
    case.bwd()
    zg = case.host("z").astype(np.float64)
    bias = orc.expand_bias(braw, wl.H_q, inp.cu_seqlens, False)
    t = tol(True)
    O, LSE = orc.dma_forward(inp.Q, inp.K, inp.V, zg, inp.cu_seqlens, wl.k, bias=bias)
    print("  O", check_close("O", case.host("O"), O, **t), flush=True)
    print("  LSE", check_close("LSE", case.host("LSE"), LSE, **t), flush=True)
    dQ, dK, dV, dz = orc.dma_backward(inp.Q, inp.K, inp.V, zg, inp.dO, inp.cu_seqlens, wl.k, bias=bias,
                                      O_stored=case.host("O"), LSE_stored=case.host("LSE"))
    for nm, ref in (("dQ", dQ), ("dK", dK), ("dV", dV), ("dz", dz)):
        print(f"  {nm}", check_close(nm, case.host(nm), ref, **t), flush=True)
    dbias = torch.full((1, inp.max_seqlen), float("nan"), device=gpu)
    B.dma_bias_bwd(case.shape, case.dz, case.cu, 1, False, dbias)
    ref_db = orc.bias_backward(dz, 1, inp.cu_seqlens, False, n_max=inp.max_seqlen)
    print("  dbias", check_close("dbias", dbias.cpu().numpy(), ref_db, **t), flush=True)
