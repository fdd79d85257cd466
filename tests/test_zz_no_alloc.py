"""calidrop_decode_static - the decode entry point that allocates nothing and takes no workspace (its
scratch is a fixed per-GPU array inside the library) - against calidrop_decode on the same inputs:
same kernels, so the results must agree bit for bit, and with the oracle to the stated tolerance.
Two calls in a row, the second with a smaller input, both in the form of the step that uses the
scratch (few (sequence, KV head) pairs, cache above 2048 rows: rows split over workgroups)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2507_19906_amd import binding as cd
from paper_2507_19906_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def prepared(lens, budget, seed, dtype="bf16", D=128):
    wl = synth.Workload(f"static_{budget}", len(lens), 8, 2, D, list(lens), 16, budget, 5, dtype, 2)
    x = {k: v.to(DEV) for k, v in synth.make_inputs(wl, seed).items()}
    bufs = H.gpu_compress(wl, x, extra_capacity=3)
    return wl, x, bufs


def decode_both_ways(wl, x, bufs, t):
    q_t = x["q_dec"][t]
    p = bufs.p
    need = cd.calidrop_decode_workspace_bytes(p, bufs.max_cache_len)
    assert 0 < need <= cd.STATIC_SCRATCH_BYTES
    bufs.decode(q_t, pass_offsets=True)                      # the existing entry point, caller's workspace
    torch.cuda.synchronize()
    want = (bufs.out.clone(), bufs.a_lse.clone(), bufs.flags.clone())
    bufs.out.zero_(); bufs.a_lse.zero_(); bufs.flags.fill_(9)
    mem = torch.cuda.memory_allocated()
    cd.calidrop_decode_static(p, q_t, bufs.k_c, bufs.v_c, bufs.cache_offsets, bufs.cache_lens, bufs.max_cache_len,
                              bufs.c_q, bufs.c_out, bufs.c_lse, bufs.out, bufs.a_lse, bufs.flags)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == mem
    assert torch.equal(bufs.out, want[0]) and torch.equal(bufs.a_lse, want[1]) and torch.equal(bufs.flags, want[2])
    rep = {}
    for b in range(wl.batch):
        H.check_decode_step(wl, bufs, q_t, b, report=rep)    # and the oracle, to the stated tolerance
    return rep


def test_static_scratch_decode_matches_the_workspace_entry_point_twice_in_a_row():
    # first call: two sequences with 5000-row caches (32 splits per head); second call: one sequence,
    # 2500 rows - it finds the first call's partials in the shared array and must not be disturbed by them
    big = prepared([9000, 7000], 5000, seed=71)
    small = prepared([4000], 2500, seed=72)
    rep1 = decode_both_ways(*big, 0)
    rep2 = decode_both_ways(*small, 0)
    rep3 = decode_both_ways(*big, 1)                          # and back to the larger shape
    print("static scratch decode:", {k: v for k, v in rep1.items() if k != "flags"},
          {k: v for k, v in rep2.items() if k != "flags"}, {k: v for k, v in rep3.items() if k != "flags"}, flush=True)


def test_static_scratch_decode_one_workgroup_form_and_fp32():
    # the form of the step that needs no scratch goes through the same entry point unchanged
    wl, x, bufs = prepared([700, 60, 900], 96, seed=73, dtype="fp32", D=64)
    decode_both_ways(wl, x, bufs, 0)
    decode_both_ways(wl, x, bufs, 1)


def test_static_scratch_decode_rejects_what_does_not_fit():
    # 150 sequences x 16 query heads with 32 splits each: more partials than the fixed array holds.
    # Refused on the host, before any HIP call, with a clear message; bad arguments are refused as by
    # calidrop_decode.
    L = cd.lib()
    A = 4096
    p = cd.make_params(dtype="bf16", batch=10, n_q_heads=128, n_kv_heads=8, head_dim=128, window=16, budget=40000,
                       pool_kernel=5)
    assert cd.calidrop_decode_workspace_bytes(p, 40000) > cd.STATIC_SCRATCH_BYTES
    rc = L.calidrop_decode_static(ctypes.byref(p), A, A, A, A, A, 40000, A, A, A, A, None, None, None)
    assert rc == cd.EWORKSPACE and "fixed array" in cd.calidrop_last_error()
    ok = cd.make_params(dtype="bf16", batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, window=16, budget=4096,
                        pool_kernel=5)
    assert L.calidrop_decode_static(ctypes.byref(ok), None, A, A, A, A, 4096, A, A, A, A, None, None, None) == cd.EINVAL
    assert L.calidrop_decode_static(ctypes.byref(ok), A, A, A + 4, A, A, 4096, A, A, A, A, None, None, None) == cd.EALIGN
    assert L.calidrop_decode_static(ctypes.byref(ok), A, A, A, A, A, 0, A, A, A, A, None, None, None) == cd.ESHAPE
