"""Seeded input generator: shapes, determinism, storage rounding."""
import numpy as np
import torch

from paper_2508_02124_amd import workloads as wlmod


def test_bf16_rounding_matches_torch_rne():
    x = np.random.default_rng(1).standard_normal(4096).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-40]      # exact ties and a denormal
    bits = wlmod.f32_to_bf16_bits(x)
    ref = torch.tensor(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (bits == ref).all()
    assert (wlmod.bf16_bits_to_f32(bits) == torch.tensor(x).to(torch.bfloat16).float().numpy()).all()


def test_cfg1_shapes_and_determinism():
    a = wlmod.make_inputs(wlmod.CONFIGS["cfg1"])
    b = wlmod.make_inputs(wlmod.CONFIGS["cfg1"])
    assert a.Q.shape == (256, 2, 64) and a.K.shape == (256, 2, 64) and a.W.shape == (2, 64)
    assert a.cu_seqlens.tolist() == [0, 256] and a.T == 256
    assert (a.Q == b.Q).all() and (a.A == b.A).all()
    assert ((a.A <= -0.5) & (a.A >= -2.0)).all()
    assert abs(float(a.W.std()) - 1 / 8) < 0.03
    f = wlmod.make_inputs(wlmod.CONFIGS["cfg1"], dtype="f32")
    assert np.abs(f.Q - a.Q).max() < 2 ** -7 * np.abs(f.Q).max()        # same draw, bf16-rounded


def test_varlen_lengths_pack_exactly():
    rng = np.random.default_rng(1005)
    lens = wlmod.draw_seqlens(rng, 65536, 512, 8192)
    assert sum(lens) == 65536 and all(1 <= n <= 8192 for n in lens)
    assert all(n >= 512 for n in lens[:-1])


def test_benchmark_shapes_follow_the_papers_speed_benchmark_table():
    """The synthetic headline and long-context workloads use the head counts, head dimension and
    precision of the paper's own kernel benchmark (fixture: tests/golden/speed_benchmark_config.txt);
    its window w = 1024 is one point of the cfg4 sweep, and bench.py warms up as often as the paper."""
    import os
    import re
    here = os.path.dirname(os.path.abspath(__file__))
    cfg = dict(line.split() for line in open(os.path.join(here, "golden", "speed_benchmark_config.txt"))
               if line.strip() and not line.startswith("#"))
    for name in ("cfg3", "cfg4"):
        wl = wlmod.CONFIGS[name]
        assert (wl.H_q, wl.H_kv, wl.d) == (int(cfg["n_h"]), int(cfg["n_h_kv"]), int(cfg["d_h"]))
    assert wlmod.CONFIGS["cfg4"].with_k(int(cfg["w"])).k == 1024
    assert wlmod.make_inputs(wlmod.CONFIGS["cfg1"]).dtype == cfg["precision"]
    bench_src = open(os.path.join(os.path.dirname(here), "bench.py")).read()
    assert re.search(r'"--warmup", type=int, default=%d\b' % int(cfg["warmups"]), bench_src)
