"""arkv_decode_step_static (split-K scratch in the library's static device array, no allocation in the call)
against arkv_decode_step on twin caches: outputs and cache contents must be identical bit for bit, on two runs in
a row, the second on a smaller cache (the array keeps the first run's contents)."""
import numpy as np
import pytest
import torch

from paper_2603_08727_amd import binding as A
from paper_2603_08727_amd import synth
from helpers import make_cfg

pytestmark = pytest.mark.gpu


def _twin_run(wl, rho, steps):
    cfg = make_cfg(wl)
    caches = [A.arkv_cache_create(cfg) for _ in range(2)]
    try:
        stats = torch.zeros((wl.batch, 3), dtype=torch.float32, device="cuda")
        k, v, qw = (t.cuda() for t in synth.prefill_inputs(wl, 0))
        scale = synth.softmax_scale(wl, 0)
        for c in caches:
            A.arkv_prefill_stats(c, 0, qw, k, wl.prefill, scale, stats)
            A.arkv_prefill_commit(c, 0, k, v, wl.prefill, np.full(wl.batch, rho, np.float32))
        q, kn, vn = (t.cuda() for t in synth.decode_inputs(wl, 0, steps))
        outs = [torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
        shape = (wl.batch, wl.n_q_heads, wl.head_dim)
        for t in range(steps):
            A.arkv_decode_step(caches[0], 0, q[t], kn[t], vn[t], scale, outs[0])
            A.arkv_decode_step_static(caches[1], 0, q[t], kn[t], vn[t], scale, outs[1])
            torch.cuda.synchronize()
            assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16)), (wl.name, t)
            f0 = A.arkv_debug_last_out_f32(caches[0], 0, shape)
            f1 = A.arkv_debug_last_out_f32(caches[1], 0, shape)
            assert np.array_equal(f0.view(np.uint32), f1.view(np.uint32)), (wl.name, t)
            assert np.isfinite(f0).all() and np.abs(f0).max() > 0
        assert A.arkv_cache_progress(caches[0], 0) == A.arkv_cache_progress(caches[1], 0)
        e0, e1 = (A.arkv_cache_export(c, 0, cfg) for c in caches)
        for name in e0:
            assert np.array_equal(e0[name], e1[name]), (wl.name, name)
        return A.arkv_cache_progress(caches[0], 0)[0]
    finally:
        for c in caches:
            A.arkv_cache_destroy(c)


def test_static_scratch_entry_point_twice_second_smaller():
    # 16 units, 4.6K live tokens each: 32 splits per unit, score folds, a tailor in the middle
    big = synth.C1.scaled(name="static_big", batch=2, n_q_heads=32, n_kv_heads=8, head_dim=128, prefill=6000,
                          budget_frac=0.8, alpha=0.98, decode_steps=130)
    n_tailors = _twin_run(big, rho=0.5, steps=130)
    assert n_tailors == 2
    # then a small cache: 2 units, 104 live tokens, one split per unit
    small = synth.C1.scaled(name="static_small", decode_steps=30)
    _twin_run(small, rho=0.5, steps=30)


def test_static_scratch_limits_are_errors():
    """More units than the array has tickets for: a clear error, nothing launched."""
    wl = synth.C1.scaled(name="static_too_big", batch=600, n_q_heads=8, n_kv_heads=8, head_dim=64, prefill=40,
                         budget_frac=2.0)
    cfg = make_cfg(wl)
    c = A.arkv_cache_create(cfg)
    try:
        k, v, qw = (t.cuda() for t in synth.prefill_inputs(wl, 0))
        stats = torch.zeros((wl.batch, 3), dtype=torch.float32, device="cuda")
        A.arkv_prefill_stats(c, 0, qw, k, wl.prefill, 0.125, stats)
        A.arkv_prefill_commit(c, 0, k, v, wl.prefill, np.ones(wl.batch, np.float32))
        q, kn, vn = (t.cuda() for t in synth.decode_inputs(wl, 0, 1))
        out = torch.zeros((wl.batch, 8, 64), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(A.ArkvError) as e:
            A.arkv_decode_step_static(c, 0, q[0], kn[0], vn[0], 0.125, out)
        assert e.value.code == A.ESCRATCH
        A.arkv_decode_step(c, 0, q[0], kn[0], vn[0], 0.125, out)      # the allocating twin still works
        torch.cuda.synchronize()
    finally:
        A.arkv_cache_destroy(c)
