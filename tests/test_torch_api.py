"""The autograd function and module over the C ABI: argument checks on the CPU; on the GPU the
output and all five gradients against the oracle (attention backward plus the chain rule of the
content scores, with the two dV parts summed)."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2508_02124_amd import binding as B
from paper_2508_02124_amd import torch_api, workloads as wlmod


def test_cpu_tensors_are_refused():
    q = torch.zeros(8, 2, 64, dtype=torch.bfloat16)
    kv = torch.zeros(8, 1, 64, dtype=torch.bfloat16)
    W, A = torch.zeros(2, 64), torch.zeros(2)
    cu = torch.tensor([0, 8], dtype=torch.int32)
    with pytest.raises(RuntimeError, match="no CPU path"):
        torch_api.dynamic_mask_attention(q, kv, kv, W, A, cu, 4)


def test_module_argument_checks():
    with pytest.raises(ValueError):
        torch_api.DynamicMaskAttention(6, 4, 64, 16)
    m = torch_api.DynamicMaskAttention(4, 2, 64, 16)
    assert m.W.shape == (4, 64) and m.A.shape == (4,) and m.W.requires_grad and m.A.requires_grad
    with pytest.raises(ValueError, match="cu_seqlens"):
        m(torch.zeros(8, 4, 64), torch.zeros(8, 2, 64), torch.zeros(8, 2, 64))


CASES = {
    # name: (seed, H_q, H_kv, d, k, seqlens)
    "gqa_d128": (31, 4, 2, 128, 96, (300, 85)),
    "mha_d64": (32, 2, 2, 64, 40, (517,)),
    "gqa_d256": (33, 4, 2, 256, 70, (290, 130)),
}


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("name", list(CASES))
def test_function_against_oracle(gpu, name, dtype):
    print(f"[case] autograd {name} {dtype}", flush=True)
    from gpu_harness import check_close, tol
    seed, H_q, H_kv, d, k, seqlens = CASES[name]
    inp = wlmod.make_inputs(wlmod.small_workload(name, seed, H_q, H_kv, d, k, seqlens), dtype=dtype)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x)).to(gpu).to(dt)
    Q, K, V = (dev(getattr(inp, n), tdt).requires_grad_() for n in "QKV")
    W, A = dev(inp.W, torch.float32).requires_grad_(), dev(inp.A, torch.float32).requires_grad_()
    cu = dev(inp.cu_seqlens.astype(np.int32), torch.int32)
    dO = dev(inp.dO, tdt)
    O = torch_api.dynamic_mask_attention(Q, K, V, W, A, cu, k, inp.max_seqlen)
    O.backward(dO)
    torch.cuda.synchronize()

    # the scores the selection was made on: the same kernel once more, through the plain binding
    shape = B.make_shape(inp.T, len(seqlens), H_q, H_kv, d, k, dtype=B.DMA_BF16 if dtype == "bf16" else B.DMA_F32,
                         max_seqlen=inp.max_seqlen)
    z = torch.empty((H_q, inp.T), dtype=torch.float32, device=gpu)
    e = torch.empty((H_q, inp.T), dtype=torch.int32, device=gpu)
    plan = torch.empty(B.dma_mask_bytes(shape), dtype=torch.uint8, device=gpu)
    B.dma_mask_gen(shape, V.detach(), W.detach(), A.detach(), cu, z, e, None, plan)
    zg = z.cpu().numpy().astype(np.float64)

    rO, _ = orc.dma_forward(inp.Q, inp.K, inp.V, zg, inp.cu_seqlens, k)
    host = lambda x: x.detach().float().cpu().numpy()
    # bf16: the backward forms D_i from the stored bf16 O (Alg. 2), so the oracle is given that buffer
    rdQ, rdK, rdV, rdz = orc.dma_backward(inp.Q, inp.K, inp.V, zg, inp.dO, inp.cu_seqlens, k,
                                          O_stored=host(O) if dtype == "bf16" else None)
    rdW, rdA, rdVz = orc.mask_backward(inp.V, inp.W, inp.A, rdz, H_q)
    t = tol(dtype == "bf16")
    print("  O", check_close("O", host(O), rO, **t), flush=True)
    print("  dQ", check_close("dQ", host(Q.grad), rdQ, **t), flush=True)
    print("  dK", check_close("dK", host(K.grad), rdK, **t), flush=True)
    print("  dV", check_close("dV", host(V.grad), rdV + rdVz, **t), flush=True)
    # dW, dA: fp32 sums over all tokens of dz * (fp32 factors), fp32 atomics, fp32 exp / log: 1e-4
    # in the fp32 path; in the bf16 path dz itself is exact to fp32 rounding (it never passes through
    # the matrix cores), so dW and dA meet the plain bf16 tolerance
    t32 = t if dtype == "bf16" else dict(atol=1e-4, rtol=1e-4, frob=1e-4)
    print("  dW", check_close("dW", host(W.grad), rdW, **t32), flush=True)
    print("  dA", check_close("dA", host(A.grad), rdA, **t32), flush=True)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_function_cross_head_against_oracle(gpu, dtype):
    """W of shape [H_q, H_kv * d]: scores from the full sampling tensor, gradients through its chain rule."""
    print(f"[case] autograd cross-head {dtype}", flush=True)
    from gpu_harness import check_close, tol
    H_q, H_kv, d, k = 4, 2, 64, 50
    inp = wlmod.make_inputs(wlmod.small_workload("xh_auto", 33, H_q, H_kv, d, k, (260, 75)), dtype=dtype)
    r = np.random.default_rng(9)
    Delta = (r.standard_normal((H_q, H_kv * d)) / np.sqrt(H_kv * d)).astype(np.float32)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x)).to(gpu).to(dt)
    Q, K, V = (dev(getattr(inp, n), tdt).requires_grad_() for n in "QKV")
    W, A = dev(Delta, torch.float32).requires_grad_(), dev(inp.A, torch.float32).requires_grad_()
    cu = dev(inp.cu_seqlens.astype(np.int32), torch.int32)
    O = torch_api.dynamic_mask_attention(Q, K, V, W, A, cu, k, inp.max_seqlen)
    O.backward(dev(inp.dO, tdt))
    torch.cuda.synchronize()
    shape = B.make_shape(inp.T, 2, H_q, H_kv, d, k, dtype=B.DMA_BF16 if dtype == "bf16" else B.DMA_F32)
    z = torch.empty((H_q, inp.T), dtype=torch.float32, device=gpu)
    B.dma_scores_xhead(shape, V.detach(), W.detach(), A.detach(), z)    # the scores the selection was made on
    zg = z.cpu().numpy().astype(np.float64)
    assert (np.abs(zg - orc.z_scores_xhead(inp.V, Delta, inp.A)) / zg).max() <= 1e-5
    rO, _ = orc.dma_forward(inp.Q, inp.K, inp.V, zg, inp.cu_seqlens, k)
    host = lambda x: x.detach().float().cpu().numpy()
    rdQ, rdK, rdV, rdz = orc.dma_backward(inp.Q, inp.K, inp.V, zg, inp.dO, inp.cu_seqlens, k,
                                          O_stored=host(O) if dtype == "bf16" else None)
    rdD, rdA, rdVz = orc.xhead_backward(inp.V, Delta, inp.A, rdz)
    t = tol(dtype == "bf16")
    print("  O", check_close("O", host(O), rO, **t), flush=True)
    print("  dQ", check_close("dQ", host(Q.grad), rdQ, **t), flush=True)
    print("  dK", check_close("dK", host(K.grad), rdK, **t), flush=True)
    print("  dV", check_close("dV", host(V.grad), rdV + rdVz, **t), flush=True)
    tw = t if dtype == "bf16" else dict(atol=1e-4, rtol=1e-4, frob=1e-4)
    print("  dDelta", check_close("dDelta", host(W.grad), rdD, **tw), flush=True)
    print("  dA", check_close("dA", host(A.grad), rdA, **tw), flush=True)


@pytest.mark.gpu
def test_module_batched_and_packed_agree(gpu):
    print("[case] autograd module", flush=True)
    torch.manual_seed(5)
    m = torch_api.DynamicMaskAttention(4, 2, 64, 32, device=gpu)
    Bsz, L = 3, 200
    q = torch.randn(Bsz, L, 4, 64, device=gpu, dtype=torch.bfloat16)
    k = torch.randn(Bsz, L, 2, 64, device=gpu, dtype=torch.bfloat16)
    v = torch.randn(Bsz, L, 2, 64, device=gpu, dtype=torch.bfloat16)
    o4 = m(q, k, v)
    cu = torch.arange(0, (Bsz + 1) * L, L, dtype=torch.int32, device=gpu)
    o3 = m(q.view(-1, 4, 64), k.view(-1, 2, 64), v.view(-1, 2, 64), cu_seqlens=cu, max_seqlen=L)
    assert o4.shape == q.shape and torch.equal(o4.view(-1, 4, 64), o3)
    o4.float().square().sum().backward()
    assert m.W.grad is not None and m.A.grad is not None
    assert torch.isfinite(m.W.grad).all() and torch.isfinite(m.A.grad).all()
    assert m.W.grad.abs().max() > 0
