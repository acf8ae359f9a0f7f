"""ctypes binding of the C-ABI library declared in include/dma.h.

Argument marshalling only: tensors (anything with .data_ptr()) or raw integer
device addresses go in, status codes come back as exceptions.  Every step of the
path runs in the HIP kernels of libdma_hip.so; if the library is missing this
module raises -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdma_hip.so")

DMA_BF16, DMA_F32 = 0, 1
DMA_OK, DMA_EINVAL, DMA_EUNSUPPORTED, DMA_EWORKSPACE, DMA_EHIP = 0, -1, -2, -3, -4


class DmaShape(ctypes.Structure):
    _fields_ = [
        ("T", ctypes.c_int32), ("n_docs", ctypes.c_int32), ("max_seqlen", ctypes.c_int32),
        ("H_q", ctypes.c_int32), ("H_kv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("k", ctypes.c_int32), ("causal", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float),
    ]


class DmaMaskLayout(ctypes.Structure):
    _fields_ = [
        ("block_rows", ctypes.c_int32), ("group_cols", ctypes.c_int32), ("max_partial", ctypes.c_int32),
        ("nblk_cap", ctypes.c_int32), ("kpad", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("off_header", ctypes.c_uint64), ("off_zq", ctypes.c_uint64), ("off_blocks", ctypes.c_uint64),
        ("off_slot_table", ctypes.c_uint64), ("off_partial_count", ctypes.c_uint64),
        ("off_partial_list", ctypes.c_uint64), ("total", ctypes.c_uint64),
    ]


class DmaError(RuntimeError):
    def __init__(self, status, what):
        super().__init__(f"{what}: {strerror(status)} (status {status})")
        self.status = status


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        shp = ctypes.POINTER(DmaShape)
        L.dma_mask_bytes.argtypes = [shp]
        L.dma_mask_bytes.restype = sz
        L.dma_workspace_bytes.argtypes = [shp]
        L.dma_workspace_bytes.restype = sz
        L.dma_mask_describe.argtypes = [shp, ctypes.POINTER(DmaMaskLayout)]
        L.dma_mask_describe.restype = i32
        L.dma_mask_gen.argtypes = [shp] + [vp] * 9
        L.dma_mask_gen.restype = i32
        L.dma_mask_gen_bias.argtypes = [shp] + [vp] * 5 + [i32, i32] + [vp] * 5
        L.dma_mask_gen_bias.restype = i32
        L.dma_bias_bwd.argtypes = [shp, vp, vp, i32, i32, vp, vp]
        L.dma_bias_bwd.restype = i32
        L.dma_fwd.argtypes = [shp] + [vp] * 10 + [sz, vp]
        L.dma_fwd.restype = i32
        L.dma_bwd.argtypes = [shp] + [vp] * 15 + [sz, vp]
        L.dma_bwd.restype = i32
        L.dma_mask_bwd.argtypes = [shp] + [vp] * 7 + [i32, vp]
        L.dma_mask_bwd.restype = i32
        L.dma_scores_xhead.argtypes = [shp] + [vp] * 5
        L.dma_scores_xhead.restype = i32
        L.dma_scores_xhead_bwd.argtypes = [shp] + [vp] * 7 + [i32, vp]
        L.dma_scores_xhead_bwd.restype = i32
        L.dma_decode_kept_bytes.argtypes = [shp]
        L.dma_decode_kept_bytes.restype = sz
        L.dma_decode.argtypes = [shp] + [vp] * 8 + [sz, vp]
        L.dma_decode.restype = i32
        L.dma_decode_static_scratch_bytes.argtypes = [shp]
        L.dma_decode_static_scratch_bytes.restype = sz
        L.dma_decode_static.argtypes = [shp] + [vp] * 9
        L.dma_decode_static.restype = i32
        L.dma_decode_step.argtypes = [shp] + [vp] * 6 + [i32] + [vp] * 3 + [sz, vp]
        L.dma_decode_step.restype = i32
        L.dma_profile_events.argtypes = [vp]
        L.dma_profile_events.restype = None
        L.dma_strerror.argtypes = [i32]
        L.dma_strerror.restype = ctypes.c_char_p
        L.dma_version.argtypes = []
        L.dma_version.restype = i32
        _lib = L
    return _lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    return ctypes.c_void_p(x.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def make_shape(T, n_docs, H_q, H_kv, d, k, causal=True, dtype=DMA_BF16, softmax_scale=0.0, max_seqlen=0):
    return DmaShape(int(T), int(n_docs), int(max_seqlen), int(H_q), int(H_kv), int(d), int(k),
                    1 if causal else 0, int(dtype), float(softmax_scale))


def strerror(status):
    return lib().dma_strerror(int(status)).decode()


def dma_version():
    return int(lib().dma_version())


STAGES = ("z", "sort", "expiry", "plan", "fwd", "bwd_zero", "bwd_dq", "bwd_dkv", "bwd_part", "bwd_cvt")


def dma_profile_events(events):
    """events: a ctypes array of 2 * len(STAGES) hipEvent_t handles (c_void_p), or None."""
    lib().dma_profile_events(events)


def dma_mask_bytes(shape):
    return int(lib().dma_mask_bytes(ctypes.byref(shape)))


def dma_workspace_bytes(shape):
    return int(lib().dma_workspace_bytes(ctypes.byref(shape)))


def dma_mask_describe(shape):
    """The layout of the mask plan (a DmaMaskLayout) for this shape."""
    out = DmaMaskLayout()
    _check(lib().dma_mask_describe(ctypes.byref(shape), ctypes.byref(out)), "dma_mask_describe")
    return out


def _check(status, what):
    if status != DMA_OK:
        raise DmaError(status, what)


def dma_mask_gen(shape, V, W, A, cu_seqlens, z, expiry, topk_idx, mask, stream=None):
    _check(lib().dma_mask_gen(ctypes.byref(shape), _ptr(V), _ptr(W), _ptr(A), _ptr(cu_seqlens), _ptr(z),
                              _ptr(expiry), _ptr(topk_idx), _ptr(mask), _stream(stream)), "dma_mask_gen")


def dma_mask_gen_bias(shape, V, W, A, cu_seqlens, bias, bias_heads, bias_per_token, z, expiry, topk_idx, mask,
                      stream=None):
    _check(lib().dma_mask_gen_bias(ctypes.byref(shape), _ptr(V), _ptr(W), _ptr(A), _ptr(cu_seqlens), _ptr(bias),
                                   int(bias_heads), int(bool(bias_per_token)), _ptr(z), _ptr(expiry), _ptr(topk_idx),
                                   _ptr(mask), _stream(stream)), "dma_mask_gen_bias")


def dma_bias_bwd(shape, dz, cu_seqlens, bias_heads, bias_per_token, dbias, stream=None):
    _check(lib().dma_bias_bwd(ctypes.byref(shape), _ptr(dz), _ptr(cu_seqlens), int(bias_heads),
                              int(bool(bias_per_token)), _ptr(dbias), _stream(stream)), "dma_bias_bwd")


def dma_fwd(shape, Q, K, V, z, expiry, mask, cu_seqlens, O, LSE, ws, ws_bytes, stream=None):
    _check(lib().dma_fwd(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(z), _ptr(expiry), _ptr(mask),
                         _ptr(cu_seqlens), _ptr(O), _ptr(LSE), _ptr(ws), int(ws_bytes), _stream(stream)), "dma_fwd")


def dma_decode_kept_bytes(shape):
    return int(lib().dma_decode_kept_bytes(ctypes.byref(shape)))


def dma_decode(shape, q, K, V, z, cu_seqlens, o, lse, kept, kept_bytes, stream=None):
    _check(lib().dma_decode(ctypes.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(z), _ptr(cu_seqlens), _ptr(o),
                            _ptr(lse), _ptr(kept), int(kept_bytes), _stream(stream)), "dma_decode")


def dma_decode_static_scratch_bytes(shape):
    return int(lib().dma_decode_static_scratch_bytes(ctypes.byref(shape)))


def dma_decode_static(shape, q, K, V, z, cu_seqlens, o, lse, kept, stream=None):
    _check(lib().dma_decode_static(ctypes.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(z), _ptr(cu_seqlens),
                                   _ptr(o), _ptr(lse), _ptr(kept), _stream(stream)), "dma_decode_static")


def dma_decode_step(shape, q, K, V, z, cu_seqlens, seq_lens, refresh, o, lse, kept, kept_bytes, stream=None):
    _check(lib().dma_decode_step(ctypes.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(z), _ptr(cu_seqlens),
                                 _ptr(seq_lens), int(bool(refresh)), _ptr(o), _ptr(lse), _ptr(kept), int(kept_bytes),
                                 _stream(stream)), "dma_decode_step")


def dma_mask_bwd(shape, V, W, A, dz, dW, dA, dV, accumulate, stream=None):
    _check(lib().dma_mask_bwd(ctypes.byref(shape), _ptr(V), _ptr(W), _ptr(A), _ptr(dz), _ptr(dW), _ptr(dA), _ptr(dV),
                              int(bool(accumulate)), _stream(stream)), "dma_mask_bwd")


def dma_scores_xhead(shape, V, Delta, A, z, stream=None):
    _check(lib().dma_scores_xhead(ctypes.byref(shape), _ptr(V), _ptr(Delta), _ptr(A), _ptr(z), _stream(stream)),
           "dma_scores_xhead")


def dma_scores_xhead_bwd(shape, V, Delta, A, dz, dDelta, dA, dV, accumulate, stream=None):
    _check(lib().dma_scores_xhead_bwd(ctypes.byref(shape), _ptr(V), _ptr(Delta), _ptr(A), _ptr(dz), _ptr(dDelta),
                                      _ptr(dA), _ptr(dV), int(bool(accumulate)), _stream(stream)),
           "dma_scores_xhead_bwd")


def dma_bwd(shape, Q, K, V, O, dO, LSE, z, expiry, mask, cu_seqlens, dQ, dK, dV, dz, ws, ws_bytes, stream=None):
    _check(lib().dma_bwd(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(z),
                         _ptr(expiry), _ptr(mask), _ptr(cu_seqlens), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dz),
                         _ptr(ws), int(ws_bytes), _stream(stream)), "dma_bwd")
