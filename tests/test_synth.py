"""The seeded input generator: shapes, determinism and the structure the recipe promises."""
import numpy as np
import torch

from paper_2507_19906_amd import synth


def test_config1_shapes_and_determinism():
    wl = synth.config(1)
    a = synth.make_inputs(wl)
    b = synth.make_inputs(wl)
    assert a["q_win"].shape == (1, 8, 16, 64) and a["q_win"].dtype == torch.float32
    assert a["q_dec"].shape == (16, 1, 8, 64)
    assert a["k"].numel() == 512 * 2 * 64 and a["seq_offsets"].tolist() == [0, 512]
    for key in a:
        assert torch.equal(a[key], b[key])


def test_structure_heavy_hitters_sink_and_ar1():
    wl = synth.config(2)
    wl.seq_lens = [2048]
    x = synth.make_inputs(wl)
    assert x["k"].dtype == torch.bfloat16
    K = synth.seq_view(x["k"], wl, 0).float()
    norms = K.norm(dim=-1)                                     # [Hkv][n]
    base = norms[:, 100:].median().item()
    assert np.all((norms[:, 0] / base).numpy() > 4.5)          # sink row x6
    heavy = (norms[:, 1:2048 - 32] > 3.0 * base).sum(dim=1)
    assert torch.all(heavy == 8)                               # 8 heavy hitters per KV head
    q = torch.cat([x["q_win"].float().permute(2, 0, 1, 3), x["q_dec"].float()])  # [w+T][b][Hq][D]
    cos = torch.nn.functional.cosine_similarity(q[1:], q[:-1], dim=-1)
    assert 0.85 < cos.mean().item() < 0.95                     # neighbour cosine ~ rho


def test_varlen_config4():
    wl = synth.config(4, batch=3)
    assert len(wl.seq_lens) == 3 and all(4096 <= n <= 16384 for n in wl.seq_lens)
    assert wl.seq_lens == synth.config(4, batch=3).seq_lens
