"""The allocation-free entry point (ccs_module_forward_static: the kernels' workspace is an array
inside the library's code object) against ccs_module_forward with a caller workspace: same kernels,
so the outputs and the appended cache rows must agree bit for bit.  Two calls in a row share the
array, the second with a smaller batch; a batch that does not fit is rejected."""
import sys

import numpy as np
import pytest
import torch

import harness as U
import workloads
from paper_2507_18006_amd import binding as B

pytestmark = pytest.mark.gpu
C = workloads.CONFIGS


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def both_ways(m, cfg, inp):
    """(y, k, v) through forward and through forward_static, each on its own buffers."""
    outs = []
    for static in (False, True):
        db = U.DeviceBatch(m, cfg, inp)
        (m.forward_static if static else m.forward)(0, db.batch)
        m.sync()
        k, v = getattr(db, "k", None), getattr(db, "v", None)
        outs.append((db.out(), None if k is None else k.float().cpu().numpy(), None if v is None else v.float().cpu().numpy()))
    return outs


def test_static_workspace_forward_equals_forward_on_two_calls_in_a_row():
    assert B.lib().ccs_static_workspace_bytes() == 64 * 1024 * 1024
    big = workloads.scaled(C["C2"], n_seqs=32, len_lo=100, len_hi=1024)       # the 7B decode step, ragged lengths
    small = workloads.scaled(big, n_seqs=5, len_lo=0, len_hi=300)             # fewer sequences, shorter caches
    w = workloads.make_weights(big, 0)
    m = U.make_module(big, w)
    try:
        for cfg, seed in ((big, 0), (small, 3)):
            say(f"[case] forward_static vs forward: {cfg.n_seqs} sequences, lens {cfg.len_lo}..{cfg.len_hi}")
            inp = workloads.make_inputs(cfg, seed)
            (y0, k0, v0), (y1, k1, v1) = both_ways(m, cfg, inp)
            assert np.isfinite(y1).all()
            assert np.array_equal(y0, y1), "outputs differ"
            assert np.array_equal(k0, k1) and np.array_equal(v0, v1), "appended cache rows differ"
            ref = U.oracle_forward(cfg, seed, w, inp)
            err = U.rel_err(y1, ref)
            say(f"  rel_err vs oracle = {err:.3e}")
            assert err <= 2e-2
    finally:
        m.destroy()


def test_static_workspace_projection_and_prefill_and_too_large_batches():
    lin = workloads.scaled(C["C5"], n_seqs=300)
    w = workloads.make_weights(lin, 1)
    m = U.make_module(lin, w, max_seqs=4096)
    try:
        for n, seed in ((300, 1), (17, 2)):           # LDS-tiled with its K split, then weight-streaming
            cfg = workloads.scaled(lin, n_seqs=n)
            say(f"[case] forward_static projection rows={n}")
            inp = workloads.make_inputs(cfg, seed)
            (y0, _, _), (y1, _, _) = both_ways(m, cfg, inp)
            assert np.array_equal(y0, y1)
        cfg = workloads.scaled(lin, n_seqs=4096)      # 4096 x 11008 packed rows alone are 90 MB
        db = U.DeviceBatch(m, cfg, workloads.make_inputs(cfg, 3))
        with pytest.raises(B.CcsError) as e:
            m.forward_static(0, db.batch)
        assert e.value.status == B.CCS_ENOMEM and "static" in str(e.value)
        m.forward(0, db.batch)                        # the caller's workspace still takes it
        m.sync()
    finally:
        m.destroy()
    pre = workloads.scaled(C["C3"], hidden=1024, n_q_heads=8, n_kv_heads=4, intermediate=2752,
                           n_seqs=5, seq_pad=80, len_lo=17, len_hi=80)
    m = U.make_module(pre, workloads.make_weights(pre, 4), seed=4)
    try:
        say("[case] forward_static prefill")
        inp = workloads.make_inputs(pre, 4)
        (y0, _, _), (y1, _, _) = both_ways(m, pre, inp)
        assert np.array_equal(y0, y1)
    finally:
        m.destroy()
