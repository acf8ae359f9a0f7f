"""The C-ABI libraries: they load, export every symbol include/*.h declares, size their buffers, and
reject bad arguments before launching anything (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2508_02124_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return B.lib()


def declared_symbols(header="dma.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dma_[a-z_]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = declared_symbols()
    assert {"dma_mask_gen", "dma_fwd", "dma_bwd", "dma_mask_bwd", "dma_decode", "dma_decode_kept_bytes",
            "dma_scores_xhead", "dma_scores_xhead_bwd", "dma_decode_step", "dma_decode_static", "dma_mask_describe",
            "dma_mask_gen_bias", "dma_bias_bwd", "dma_profile_events",
            "dma_mask_bytes", "dma_workspace_bytes",
            "dma_strerror", "dma_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert B.dma_version() >= 100
    assert not any("probe" in n for n in names)          # the benchmark's yardsticks are not in the product library
    assert not hasattr(lib, "dma_probe_mfma")


def test_probe_header_symbols_exported(lib):
    """include/dma_probe.h <-> libdma_probe.so; every header under include/ is covered by one of these tests."""
    from paper_2508_02124_amd import probe as P
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["dma.h", "dma_probe.h"]
    names = declared_symbols("dma_probe.h")
    assert names == ["dma_probe_copy", "dma_probe_mfma"]
    for n in names:
        assert hasattr(P.lib(), n), n
    p = 0x1000
    with pytest.raises(B.DmaError) as e:
        P.dma_probe_copy(p, p + 8, 1024, stream=0)       # misaligned: refused before any launch
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        P.dma_probe_mfma(None, 4, 4, stream=0)
    assert e.value.status == B.DMA_EINVAL


def test_sizes_and_shape_validation(lib):
    s = B.make_shape(T=16384, n_docs=1, H_q=32, H_kv=8, d=128, k=2048)
    mb, wb = B.dma_mask_bytes(s), B.dma_workspace_bytes(s)
    assert mb > 32 * 129 * 2048 * 4            # at least the slot table
    assert wb >= 32 * 16384 * 4 + 2 * 16384 * 8 * 128 * 4
    for bad in (dict(T=0), dict(k=0), dict(H_kv=3), dict(n_docs=0)):
        kw = dict(T=256, n_docs=1, H_q=4, H_kv=2, d=64, k=16)
        kw.update(bad)
        assert B.dma_mask_bytes(B.make_shape(**kw)) == 0
    assert B.dma_mask_bytes(B.make_shape(T=256, n_docs=1, H_q=4, H_kv=2, d=96, k=16)) == 0
    f32 = B.make_shape(T=256, n_docs=1, H_q=2, H_kv=2, d=64, k=64, dtype=B.DMA_F32)
    assert B.dma_workspace_bytes(f32) >= 2 * 256 * 4


def test_error_codes_before_any_launch(lib):
    ok = B.make_shape(T=256, n_docs=1, H_q=2, H_kv=2, d=64, k=64)
    p = 0x1000                                   # aligned dummy address: never dereferenced on a failing call
    with pytest.raises(B.DmaError) as e:
        B.dma_mask_gen(ok, p, p, p, None, p, p, None, p, stream=0)       # cu_seqlens missing
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_mask_gen(ok, p, p, p, p, p + 4, p, None, p, stream=0)      # z misaligned
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_fwd(B.make_shape(T=256, n_docs=1, H_q=2, H_kv=2, d=80, k=64), p, p, p, p, p, p, p, p, p, None, 0, stream=0)
    assert e.value.status == B.DMA_EUNSUPPORTED
    assert B.dma_mask_bytes(B.make_shape(T=256, n_docs=1, H_q=2, H_kv=2, d=64, k=64, causal=False)) > 0
    with pytest.raises(B.DmaError) as e:
        B.dma_bwd(ok, p, p, p, p, p, p, p, p, p, p, p, p, p, p, p, 16, stream=0)   # workspace too small
    assert e.value.status == B.DMA_EWORKSPACE
    with pytest.raises(B.DmaError) as e:
        B.dma_bwd(ok, p, p, p, p, p, p, p, p, p, p, None, p, p, p, p, 1 << 30, stream=0)   # dQ missing
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_mask_bwd(ok, p, p, p, p, None, p, p, 0, stream=0)          # dW missing
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_mask_bwd(ok, p, p, p, p + 8, p, p, p, 1, stream=0)         # dz misaligned
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_scores_xhead(ok, p, None, p, p, stream=0)                  # Delta missing
    assert e.value.status == B.DMA_EINVAL
    many = B.make_shape(T=256, n_docs=1, H_q=64, H_kv=2, d=64, k=64)
    with pytest.raises(B.DmaError) as e:
        B.dma_scores_xhead(many, p, p, p, p, stream=0)                   # more than 32 heads
    assert e.value.status == B.DMA_EUNSUPPORTED
    with pytest.raises(B.DmaError) as e:
        B.dma_scores_xhead_bwd(many, p, p, p, p, p, p, p, 0, stream=0)
    assert e.value.status == B.DMA_EUNSUPPORTED
    with pytest.raises(B.DmaError) as e:
        B.dma_scores_xhead_bwd(ok, p, p, p, p, p + 4, p, p, 0, stream=0)  # dDelta misaligned
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_decode(ok, p, p, p, p, p, p, p, p, 0, stream=0)            # kept buffer too small
    assert e.value.status == B.DMA_EWORKSPACE
    with pytest.raises(B.DmaError) as e:
        B.dma_decode(ok, p, p, p, p, None, p, p, p, 1 << 30, stream=0)   # cu_seqlens missing
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_decode_step(ok, p, p, p, p, p, None, 1, p, p, p, 1 << 30, stream=0)   # seq_lens missing
    assert e.value.status == B.DMA_EINVAL
    with pytest.raises(B.DmaError) as e:
        B.dma_decode_step(ok, p, p, p, p, p, p, 0, p, p, p, 8, stream=0)            # kept buffer too small
    assert e.value.status == B.DMA_EWORKSPACE
    # bf16 attention addresses gathered K / V rows with 32-bit offsets: K (or V) beyond 4 GiB is refused
    huge = B.make_shape(T=1 << 23, n_docs=1, H_q=8, H_kv=8, d=128, k=64)       # 8 Mi tokens x 2 KiB = 16 GiB
    with pytest.raises(B.DmaError) as e:
        B.dma_fwd(huge, p, p, p, p, p, p, p, p, p, None, 0, stream=0)
    assert e.value.status == B.DMA_EUNSUPPORTED
    with pytest.raises(B.DmaError) as e:
        B.dma_bwd(huge, p, p, p, p, p, p, p, p, p, p, p, p, p, p, p, 1 << 62, stream=0)
    assert e.value.status == B.DMA_EUNSUPPORTED
    # the score kernel keeps a group's projection vectors in LDS: more than 256 q-heads per kv-head is refused
    wide = B.make_shape(T=256, n_docs=1, H_q=257, H_kv=1, d=64, k=64)
    assert B.dma_mask_bytes(wide) == 0
    with pytest.raises(B.DmaError) as e:
        B.dma_mask_gen(wide, p, p, p, p, p, p, None, p, stream=0)
    assert e.value.status == B.DMA_EUNSUPPORTED
    # the score-gradient kernel keeps a token tile and the group's vectors in LDS: a group too large for it
    # is refused before the first launch
    big_group = B.make_shape(T=256, n_docs=1, H_q=64, H_kv=1, d=128, k=64)
    with pytest.raises(B.DmaError) as e:
        B.dma_mask_bwd(big_group, p, p, p, p, p, p, p, 0, stream=0)
    assert e.value.status == B.DMA_EUNSUPPORTED
    # head dimension 256: everything but the cross-head scores takes it
    wide_d = B.make_shape(T=256, n_docs=1, H_q=2, H_kv=2, d=256, k=64)
    assert B.dma_mask_bytes(wide_d) > 0 and B.dma_workspace_bytes(wide_d) > 0
    with pytest.raises(B.DmaError) as e:
        B.dma_scores_xhead(wide_d, p, p, p, p, stream=0)
    assert e.value.status == B.DMA_EUNSUPPORTED
    assert B.dma_decode_kept_bytes(wide_d) >= 2 * 64 * 4
    assert B.dma_decode_kept_bytes(ok) >= 2 * 64 * 4
    assert "workspace" in B.strerror(B.DMA_EWORKSPACE)
    assert B.strerror(0) == "ok"
