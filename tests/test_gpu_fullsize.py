"""Full-size workloads in the launch configuration the benchmark times, checked on sampled
(sequence, KV head) pairs that the oracle can afford.  Needs an MI355X."""
import numpy as np
import pytest
import torch

from paper_2507_19906_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def sampled(wl, samples, decode_steps=2, seed=synth.BASE_SEED):
    x = synth.make_inputs(wl, seed, device=DEV)
    bufs = H.gpu_compress(wl, x)
    rep = {}
    for b, g in samples:
        H.check_compress(wl, x, bufs, b, heads=[g], report=rep)
    for t in range(decode_steps):
        bufs.decode(x["q_dec"][t])
        torch.cuda.synchronize()
        for b, g in samples:
            H.check_decode_step(wl, bufs, x["q_dec"][t], b, heads=[g], report=rep)
    # properties that hold for every (sequence, head), checked on all of them
    idx = bufs.indices.cpu().numpy()
    for b, n in enumerate(wl.seq_lens):
        L = min(wl.budget, n)
        assert int(bufs.cache_lens[b]) == L
        assert np.all(np.diff(idx[b, :, :L], axis=1) > 0)
        if n > wl.budget:
            assert np.array_equal(idx[b, :, L - wl.window:L],
                                  np.tile(np.arange(n - wl.window, n), (wl.n_kv_heads, 1)))
            assert np.all(idx[b, :, 0] >= 0) and np.all(idx[b, :, L - 1] == n - 1)
    assert torch.isfinite(bufs.c_out).all() and torch.isfinite(bufs.out.float()).all()
    print(wl.name, {k: (v if k != "flags" else np.bincount(v, minlength=3).tolist()) for k, v in rep.items()},
          flush=True)
    return rep


def test_config3_stack_32_layers_budget_512():
    wl = synth.config(3, layers=32, budget=512, decode_steps=2)
    sampled(wl, [(0, 1), (31, 6), (13, 0), (22, 7)])


@pytest.mark.parametrize("budget", [128, 2048])
def test_config3_other_budgets(budget):
    wl = synth.config(3, layers=8, budget=budget, decode_steps=2)
    sampled(wl, [(5, 3), (0, 0)])


def test_config4_batch64_varlen():
    wl = synth.config(4, decode_steps=2)
    lens = wl.seq_lens
    b_short, b_long = int(np.argmin(lens)), int(np.argmax(lens))
    sampled(wl, [(b_short, 0), (b_long, 7), (17, 4)])


def test_config5_long_context_131k():
    wl = synth.config(5, decode_steps=2)
    sampled(wl, [(0, 2)])
