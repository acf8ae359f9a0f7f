"""Device-resident buffers of one workload and the calls of the hot path on them.

Plumbing shared by the benchmark, the smoke check and the GPU tests: it allocates the inputs and
outputs of dma_mask_gen / dma_fwd / dma_bwd with torch (device memory only) and calls the C ABI
through the binding.  No arithmetic of the method happens here.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import workloads as wlmod


def to_dev(x, dev, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(dev)


def bf16_tensor_from_f32(x, dev):
    """fp32 / fp64 array -> device bf16 tensor, rounded to nearest even on the host (bit-exact with workloads)."""
    bits = wlmod.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)


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

    def set_forward_results(self, O, LSE):
        """Overwrite the O and LSE buffers that dma_bwd reads (e.g. with a reference forward result:
        O rounded to the path's storage dtype, LSE to fp32)."""
        if self.is_bf16:
            self.O.copy_(bf16_tensor_from_f32(O, self.dev))
        else:
            self.O.copy_(to_dev(np.asarray(O, dtype=np.float32), self.dev))
        self.LSE.copy_(to_dev(np.asarray(LSE, dtype=np.float32), self.dev))

    def host(self, name):
        torch.cuda.synchronize()
        t = getattr(self, name)
        return t.float().cpu().numpy() if t.is_floating_point() else t.cpu().numpy()

    def plan_views(self):
        """Host views of the mask plan's inspectable parts, located by dma_mask_describe."""
        L = B.dma_mask_describe(self.shape)
        H = self.wl.H_q
        raw = self.mask.cpu().numpy()

        def view(off, count, shape):
            return raw[off:off + 4 * count].view(np.int32).reshape(shape)
        return dict(
            block_rows=L.block_rows, group_cols=L.group_cols, max_partial=L.max_partial,
            nblk=int(view(L.off_header, 1, (1,))[0]),
            blk=view(L.off_blocks, L.nblk_cap * 4, (L.nblk_cap, 4)),
            slot=view(L.off_slot_table, H * L.nblk_cap * L.kpad, (H, L.nblk_cap, L.kpad)),
            pcnt=view(L.off_partial_count, H * L.nblk_cap, (H, L.nblk_cap)),
            plist=view(L.off_partial_list, H * L.nblk_cap * L.max_partial, (H, L.nblk_cap, L.max_partial)),
        )
