"""dma_decode_static (library-owned scratch, no allocation) against dma_decode, through the C ABI.

Two calls in a row on one stream, the second with a smaller input: the static scratch keeps the first
call's contents, so anything the kernels fail to clear would show in the second comparison.  The
results must match dma_decode's to the parity bar: kept indices bit for bit, o / lse within the
bf16 tolerance (the two entry points run the same kernels, so they are in fact identical)."""
import numpy as np
import pytest
import torch

from paper_2508_02124_amd import binding as B
from paper_2508_02124_amd import workloads as wlmod

pytestmark = pytest.mark.gpu


def _case(gpu, seed, lens, H_q, H_kv, d, k):
    r = np.random.default_rng(seed)
    T = sum(lens)
    rb = lambda shape: wlmod.bf16_bits_to_f32(wlmod.f32_to_bf16_bits(r.standard_normal(shape, dtype=np.float32)))
    dev = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x)).to(gpu).to(dt)
    z = r.uniform(0.05, 1.0, size=(H_q, T)).astype(np.float32)
    z[0] = np.round(z[0] * 16) / 16                   # ties across the threshold in one head
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return dict(shape=B.make_shape(T=T, n_docs=len(lens), H_q=H_q, H_kv=H_kv, d=d, k=k),
                q=dev(rb((len(lens), H_q, d)), torch.bfloat16), K=dev(rb((T, H_kv, d)), torch.bfloat16),
                V=dev(rb((T, H_kv, d)), torch.bfloat16), z=dev(z, torch.float32), cu=dev(cu, torch.int32),
                n=len(lens), H_q=H_q, d=d, kcap=min(k, T))


def _run_both(gpu, c):
    shape, n, H_q, d, kcap = c["shape"], c["n"], c["H_q"], c["d"], c["kcap"]
    nlist = n * H_q * kcap
    # reference entry point: kept lists + scratch in one caller buffer
    kept_a = torch.full((B.dma_decode_kept_bytes(shape) // 4,), -5, dtype=torch.int32, device=gpu)
    o_a = torch.full((n, H_q, d), float("nan"), dtype=torch.bfloat16, device=gpu)
    lse_a = torch.full((H_q, n), float("nan"), device=gpu)
    B.dma_decode(shape, c["q"], c["K"], c["V"], c["z"], c["cu"], o_a, lse_a, kept_a, kept_a.numel() * 4)
    # allocation-free entry point: the kept lists only
    kept_b = torch.full((nlist,), -5, dtype=torch.int32, device=gpu)
    o_b = torch.full((n, H_q, d), float("nan"), dtype=torch.bfloat16, device=gpu)
    lse_b = torch.full((H_q, n), float("nan"), device=gpu)
    assert 0 < B.dma_decode_static_scratch_bytes(shape) <= (4 << 20)
    before = torch.cuda.memory_allocated(gpu)
    B.dma_decode_static(shape, c["q"], c["K"], c["V"], c["z"], c["cu"], o_b, lse_b, kept_b)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated(gpu) == before
    assert torch.equal(kept_a[:nlist], kept_b), "kept sets differ"
    oa, ob = o_a.float().cpu().numpy(), o_b.float().cpu().numpy()
    la, lb = lse_a.cpu().numpy(), lse_b.cpu().numpy()
    assert np.isfinite(ob).all()
    assert (np.abs(oa - ob) <= 2e-2 + 1e-2 * np.abs(oa)).all(), np.abs(oa - ob).max()
    fin = np.isfinite(la)
    assert (fin == np.isfinite(lb)).all() and (np.abs(la[fin] - lb[fin]) <= 2e-2 + 1e-2 * np.abs(la[fin])).all()
    return float(np.abs(oa - ob).max())


def test_static_scratch_decode_matches_decode_twice(gpu):
    print("[case] dma_decode_static vs dma_decode: large call, then a smaller one", flush=True)
    big = _case(gpu, 91, (70000, 3000, 0, 517), H_q=8, H_kv=2, d=128, k=2048)
    small = _case(gpu, 92, (300, 40), H_q=4, H_kv=4, d=64, k=100)
    print("  first call  max|o diff|", _run_both(gpu, big), flush=True)
    print("  second call max|o diff|", _run_both(gpu, small), flush=True)


def test_static_scratch_decode_refuses_what_does_not_fit(gpu):
    # 64 sequences x 64 heads x k = 4096: more scratch than the library holds; refused before any launch
    shape = B.make_shape(T=1 << 20, n_docs=64, H_q=64, H_kv=8, d=128, k=4096)
    assert B.dma_decode_static_scratch_bytes(shape) > (4 << 20)
    p = 0x1000
    with pytest.raises(B.DmaError) as e:
        B.dma_decode_static(shape, p, p, p, p, p, p, p, p, stream=0)
    assert e.value.status == B.DMA_EWORKSPACE
