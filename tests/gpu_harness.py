"""Shared plumbing of the GPU parity tests: device buffers, calls through the C ABI, tolerances.

Tolerance (bf16 path): element-wise |gpu - ref| <= 2e-2 + 1e-2 |ref| and
||gpu - ref||_F <= 1e-2 ||ref||_F.  fp32 debug path: the same form with 1e-5.
"""
from __future__ import annotations

import numpy as np
import torch

from paper_2508_02124_amd import binding as B
from paper_2508_02124_amd import workloads as wlmod

BQ, SG, MAXPART = 256, 128, 512


def to_dev(x, dev, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(dev)


class DeviceCase:
    """Device-resident inputs and outputs of one workload."""

    def __init__(self, inp: wlmod.Inputs, dev, z_override=None, topk=False):
        wl = inp.wl
        self.inp, self.wl, self.dev = inp, wl, dev
        self.is_bf16 = inp.dtype == "bf16"
        tdt = torch.bfloat16 if self.is_bf16 else torch.float32
        T = inp.T
        self.T = T
        self.n_docs = len(inp.cu_seqlens) - 1
        self.shape = B.make_shape(T, self.n_docs, wl.H_q, wl.H_kv, wl.d, wl.k, causal=wl.causal,
                                  dtype=B.DMA_BF16 if self.is_bf16 else B.DMA_F32, max_seqlen=inp.max_seqlen)

        def act(name):
            if self.is_bf16:
                return torch.from_numpy(inp.bits[name].view(np.int16)).view(torch.bfloat16).to(dev)
            return to_dev(getattr(inp, name), dev)

        self.Q, self.K, self.V, self.dO = act("Q"), act("K"), act("V"), act("dO")
        self.W, self.A = to_dev(inp.W, dev), to_dev(inp.A, dev)
        self.cu = to_dev(inp.cu_seqlens.astype(np.int32), dev)
        self.z = torch.empty((wl.H_q, T), dtype=torch.float32, device=dev)
        self.z_given = z_override is not None
        if self.z_given:
            self.z.copy_(to_dev(np.asarray(z_override, dtype=np.float32), dev))
        self.expiry = torch.full((wl.H_q, T), -7, dtype=torch.int32, device=dev)
        self.topk = torch.full((wl.H_q, T, wl.k), -9, dtype=torch.int32, device=dev) if topk else None
        self.mask = torch.empty(B.dma_mask_bytes(self.shape), dtype=torch.uint8, device=dev)
        self.ws_bytes = B.dma_workspace_bytes(self.shape)
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=dev)
        self.O = torch.full((T, wl.H_q, wl.d), float("nan"), dtype=tdt, device=dev)
        self.LSE = torch.full((wl.H_q, T), float("nan"), dtype=torch.float32, device=dev)
        self.dQ = torch.full((T, wl.H_q, wl.d), float("nan"), dtype=tdt, device=dev)
        self.dK = torch.full((T, wl.H_kv, wl.d), float("nan"), dtype=tdt, device=dev)
        self.dV = torch.full((T, wl.H_kv, wl.d), float("nan"), dtype=tdt, device=dev)
        self.dz = torch.full((wl.H_q, T), float("nan"), dtype=torch.float32, device=dev)

    def mask_gen(self):
        B.dma_mask_gen(self.shape, self.V, None if self.z_given else self.W, self.A, self.cu, self.z,
                       self.expiry, self.topk, self.mask)

    def fwd(self):
        B.dma_fwd(self.shape, self.Q, self.K, self.V, self.z, self.expiry, self.mask, self.cu, self.O,
                  self.LSE, self.ws, self.ws_bytes)

    def bwd(self):
        B.dma_bwd(self.shape, self.Q, self.K, self.V, self.O, self.dO, self.LSE, self.z, self.expiry,
                  self.mask, self.cu, self.dQ, self.dK, self.dV, self.dz, self.ws, self.ws_bytes)

    def host(self, name):
        torch.cuda.synchronize()
        t = getattr(self, name)
        return t.float().cpu().numpy() if t.is_floating_point() else t.cpu().numpy()

    # ---- plan readback (mirror of the library's layout, tests only)
    def plan_views(self):
        T, H, n_docs, k = self.T, self.wl.H_q, self.n_docs, self.wl.k
        nblk_cap = T // BQ + n_docs
        kpad = (min(k, T) + SG - 1) // SG * SG
        raw = self.mask.cpu().numpy()
        o = 0

        def take(nbytes):
            nonlocal o
            r = o
            o = (o + nbytes + 255) // 256 * 256
            return r
        off_hdr = take(64)
        take(512)            # constants
        take(H * T * 4)      # z / softmax_scale
        off_blk = take(nblk_cap * 16)
        off_docblk = take((n_docs + 1) * 4)
        off_slot = take(H * nblk_cap * kpad * 4)
        off_pcnt = take(H * nblk_cap * 4)
        off_plist = take(H * nblk_cap * MAXPART * 4)

        def view(off, count, shape):
            return raw[off:off + 4 * count].view(np.int32).reshape(shape)
        return dict(
            nblk=int(view(off_hdr, 1, (1,))[0]),
            blk=view(off_blk, nblk_cap * 4, (nblk_cap, 4)),
            slot=view(off_slot, H * nblk_cap * kpad, (H, nblk_cap, kpad)),
            pcnt=view(off_pcnt, H * nblk_cap, (H, nblk_cap)),
            plist=view(off_plist, H * nblk_cap * MAXPART, (H, nblk_cap, MAXPART)),
        )


def check_close(name, got, ref, atol, rtol, frob, summand_abs=None, srel=0.0):
    """summand_abs / srel: for an output that is a long sum with cancellation (dz), the oracle's
    sum of |summands| and the relative error each summand may carry; the element-wise bound grows
    by srel * summand_abs."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values in the GPU result"
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    if summand_abs is not None:
        bound = bound + srel * np.asarray(summand_abs, dtype=np.float64)
    worst = int(np.argmax(err - bound))
    assert (err <= bound).all(), (
        f"{name}: max|err|={err.max():.3e} at flat index {worst}: gpu={got.flat[worst]:.6g} ref={ref.flat[worst]:.6g}")
    # an identically zero reference (k = 1 makes dS, dQ, dK and dz vanish) leaves the relative norm
    # undefined: below the norm of the absolute tolerance the element-wise bound alone decides
    nref = np.linalg.norm(ref)
    if nref <= atol * np.sqrt(ref.size):
        return float(err.max()), 0.0
    fr = np.linalg.norm(got - ref) / nref
    assert fr <= frob, f"{name}: relative Frobenius error {fr:.3e} > {frob}"
    return float(err.max()), float(fr)


# dz_j = sum_i dS_ij, dS_ij = P_ij (dP_ij - D_i).  In the bf16 path D_i = dO_i . O_i uses the stored
# bf16 O (as Alg. 2 does), so every summand carries a relative error of order 2^-8 that does not
# shrink with |dz_j| when the summands cancel: judge dz against 2e-2 + 1e-2 |ref| + DZ_SREL sum_i |dS_ij|.
DZ_SREL = 5e-3


# fp32 debug path: dK, dV and dz of a key are sums over the rows that keep it, accumulated one row
# after the other in fp32; judged against 1e-5 + 1e-5 |ref| + F32_SREL sum |terms| (17 ulps of the
# summand mass; it is below the plain tolerance until a key is kept by about a thousand rows).
F32_SREL = 1e-6


def dz_allowance(dz_abs, dzD):
    """summand_abs for check_close(..., srel=DZ_SREL) on dz: the sum of |dS_ij| (bf16 rounding of the
    factors of dS), plus the stored-O term: O is kept in bf16, so D_i = dO_i . O_i is off by up to
    2^-9 sum_c |dO_ic O_ic|, and that error enters dz_j weighted by P_ij whatever the size of dS_ij
    (it is what matters for short documents, where P is of order one)."""
    return np.asarray(dz_abs) + (2.0 ** -9 / DZ_SREL) * np.asarray(dzD)


def dq_allowance(dQD):
    """summand_abs for check_close(..., srel=DZ_SREL) on the bf16 dQ: the stored-O error of D_i (up to
    2^-9 sum_c |dO_ic O_ic|) enters dQ_i = scale sum_j dS_ij k_j through every kept key, weighted by
    P_ij; it only matters when a row keeps one or two keys (P of order one)."""
    return (2.0 ** -9 / DZ_SREL) * np.asarray(dQD)


def tol(is_bf16):
    return dict(atol=2e-2, rtol=1e-2, frob=1e-2) if is_bf16 else dict(atol=1e-5, rtol=1e-5, frob=1e-5)
