"""GPU tests of the C ABI beyond plain parity: the multi-layer entry point, call-order errors,
bitwise repeatability, reset and re-commit, the measurement hooks."""
import numpy as np
import pytest
import torch

from paper_2603_08727_amd import binding as A
from paper_2603_08727_amd import synth
from helpers import SideBySide, make_cfg

pytestmark = pytest.mark.gpu


def _prepare(wl, rho=0.5):
    cfg = make_cfg(wl)
    cache = A.arkv_cache_create(cfg)
    stats = torch.zeros((wl.n_layers, wl.batch, 3), dtype=torch.float32, device="cuda")
    ins = []
    for l in range(wl.n_layers):
        k, v, qw = (t.cuda() for t in synth.prefill_inputs(wl, l))
        A.arkv_prefill_stats(cache, l, qw, k, wl.prefill, synth.softmax_scale(wl, l), stats[l])
        ins.append((k, v))
    for l in range(wl.n_layers):
        A.arkv_prefill_commit(cache, l, ins[l][0], ins[l][1], wl.prefill, np.full(wl.batch, rho, np.float32))
    return cfg, cache


def _export_all(cache, cfg, L):
    return [A.arkv_cache_export(cache, l, cfg) for l in range(L)]


def test_layers_entry_point_equals_per_layer_calls():
    """arkv_decode_step_layers over 3 layers == three arkv_decode_step calls, bit for bit, through a tailor."""
    wl = synth.C1.scaled(name="multi", n_layers=3, batch=2, decode_steps=30)
    L, B = wl.n_layers, wl.batch
    cfg, c1 = _prepare(wl)
    _, c2 = _prepare(wl)
    try:
        dins = [tuple(t.cuda() for t in synth.decode_inputs(wl, l)) for l in range(L)]
        q = torch.stack([d[0] for d in dins], 1).contiguous()
        kn = torch.stack([d[1] for d in dins], 1).contiguous()
        vn = torch.stack([d[2] for d in dins], 1).contiguous()
        sc = np.array([synth.softmax_scale(wl, l) for l in range(L)], np.float32)
        o1 = torch.empty((L, B, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device="cuda")
        o2 = torch.empty_like(o1)
        for t in range(wl.decode_steps):
            for l in range(L):
                A.arkv_decode_step(c1, l, q[t, l], kn[t, l], vn[t, l], float(sc[l]), o1[l])
            A.arkv_decode_step_layers(c2, 0, L, q[t], kn[t], vn[t], sc, o2)
            assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)), t
        assert A.arkv_cache_progress(c1, 0)[0] >= 2
        for e1, e2 in zip(_export_all(c1, cfg, L), _export_all(c2, cfg, L)):
            for k in e1:
                assert np.array_equal(e1[k], e2[k]), k
    finally:
        A.arkv_cache_destroy(c1); A.arkv_cache_destroy(c2)


def test_bitwise_repeatability():
    """Two runs of the same trajectory give identical bytes (no float atomics anywhere)."""
    wl = synth.C1.scaled(name="repeat", decode_steps=40)
    outs = []
    for _ in range(2):
        cfg, c = _prepare(wl, rho=0.4)
        try:
            q, kn, vn = (t.cuda() for t in synth.decode_inputs(wl, 0))
            o = torch.empty((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device="cuda")
            acc = []
            for t in range(wl.decode_steps):
                A.arkv_decode_step(c, 0, q[t], kn[t], vn[t], synth.softmax_scale(wl, 0), o)
                acc.append(o.clone())
            outs.append((torch.stack(acc).cpu().view(torch.int16).numpy(), A.arkv_cache_export(c, 0, cfg)))
        finally:
            A.arkv_cache_destroy(c)
    assert np.array_equal(outs[0][0], outs[1][0])
    for k in outs[0][1]:
        assert np.array_equal(outs[0][1][k], outs[1][1][k]), k


def test_call_order_errors_and_reset():
    wl = synth.C1.scaled(name="order", prefill=200, decode_steps=4)
    cfg = make_cfg(wl)
    c = A.arkv_cache_create(cfg)
    try:
        k, v, qw = (t.cuda() for t in synth.prefill_inputs(wl, 0))
        q, kn, vn = (t.cuda() for t in synth.decode_inputs(wl, 0))
        o = torch.empty((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device="cuda")
        stats = torch.zeros((wl.batch, 3), dtype=torch.float32, device="cuda")
        rho = np.full(wl.batch, 0.5, np.float32)
        with pytest.raises(A.ArkvError) as e:                      # decode before commit
            A.arkv_decode_step(c, 0, q[0], kn[0], vn[0], 0.1, o)
        assert e.value.code == A.ESTATE
        with pytest.raises(A.ArkvError) as e:                      # commit before scoring
            A.arkv_prefill_commit(c, 0, k, v, wl.prefill, rho)
        assert e.value.code == A.ESTATE
        with pytest.raises(A.ArkvError) as e:                      # prompt not longer than the window
            A.arkv_prefill_stats(c, 0, qw, k, wl.window, 0.1, stats)
        assert e.value.code == A.EINVAL
        with pytest.raises(A.ArkvError) as e:                      # layer out of range
            A.arkv_prefill_stats(c, 5, qw, k, wl.prefill, 0.1, stats)
        assert e.value.code == A.EINVAL
        A.arkv_prefill_stats(c, 0, qw, k, wl.prefill, 0.1, stats)
        with pytest.raises(A.ArkvError) as e:                      # commit with another length
            A.arkv_prefill_commit(c, 0, k, v, wl.prefill - 1, rho)
        assert e.value.code == A.ESTATE
        A.arkv_prefill_commit(c, 0, k, v, wl.prefill, rho)
        with pytest.raises(A.ArkvError) as e:                      # commit twice
            A.arkv_prefill_commit(c, 0, k, v, wl.prefill, rho)
        assert e.value.code == A.ESTATE
        A.arkv_decode_step(c, 0, q[0], kn[0], vn[0], 0.1, o)
        first = A.arkv_cache_export(c, 0, cfg)
        # a new request on the same memory gives the same result
        A.arkv_cache_reset(c, 0)
        A.arkv_prefill_stats(c, 0, qw, k, wl.prefill, 0.1, stats)
        A.arkv_prefill_commit(c, 0, k, v, wl.prefill, rho)
        A.arkv_decode_step(c, 0, q[0], kn[0], vn[0], 0.1, o)
        second = A.arkv_cache_export(c, 0, cfg)
        for key in first:
            assert np.array_equal(first[key], second[key]), key
    finally:
        A.arkv_cache_destroy(c)


def test_prefill_attention_argument_errors():
    wl = synth.C1.scaled(name="attn_err", prefill=200, decode_steps=2)
    cfg = make_cfg(wl)
    c = A.arkv_cache_create(cfg)
    try:
        k, v, qw = (t.cuda() for t in synth.prefill_inputs(wl, 0))
        T, W = wl.prefill, wl.window
        q = torch.zeros((wl.batch, wl.n_q_heads, T, wl.head_dim), dtype=torch.bfloat16, device="cuda")
        out = torch.empty_like(q)
        stats = torch.zeros((wl.batch, 3), dtype=torch.float32, device="cuda")
        for args in [(0, T + 1, T, 0.1, None),        # more queries than keys
                     (0, 0, T, 0.1, None),            # no query
                     (0, T, T, 0.0, None),            # scale must be positive
                     (3, T, T, 0.1, None),            # layer out of range
                     (0, W - 1, T, 0.1, stats),       # the scorer needs the whole window among the queries
                     (0, W, W, 0.1, stats)]:          # ... and a prompt longer than the window
            layer, Tq, Tk, scale, st = args
            with pytest.raises(A.ArkvError) as e:
                A.arkv_prefill_attention(c, layer, q[:, :, :max(Tq, 1)].contiguous(), k, v, Tq, Tk, scale, out, st)
            assert e.value.code == A.EINVAL, args
        lse = torch.zeros((wl.batch, wl.n_q_heads, W), dtype=torch.float32, device="cuda")
        for layer, Tk, scale in [(3, T, 0.1), (0, W, 0.1), (0, T, -1.0)]:   # the log-sum-exp variant checks the same
            with pytest.raises(A.ArkvError) as e:
                A.arkv_prefill_stats_lse(c, layer, qw, k, Tk, scale, lse, stats)
            assert e.value.code == A.EINVAL
        A.arkv_prefill_attention(c, 0, q, k, v, T, T, 0.1, out, stats)      # scores the layer
        A.arkv_prefill_commit(c, 0, k, v, T, np.full(wl.batch, 0.5, np.float32))
        with pytest.raises(A.ArkvError) as e:
            A.arkv_prefill_stats_lse(c, 0, qw, k, T, 0.1, lse, stats)
        assert e.value.code == A.ESTATE
        with pytest.raises(A.ArkvError) as e:                               # scoring a committed layer again
            A.arkv_prefill_attention(c, 0, q, k, v, T, T, 0.1, out, stats)
        assert e.value.code == A.ESTATE
        A.arkv_prefill_attention(c, 0, q, k, v, T, T, 0.1, out, None)       # attention alone is still allowed
        torch.cuda.synchronize()
    finally:
        A.arkv_cache_destroy(c)


def test_measurement_hooks():
    wl = synth.C1.scaled(name="hooks", decode_steps=6)
    cfg, c = _prepare(wl)
    try:
        q, kn, vn = (t.cuda() for t in synth.decode_inputs(wl, 0))
        o = torch.empty((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device="cuda")
        A.arkv_debug_time_attend(c, True)
        for t in range(wl.decode_steps):
            A.arkv_decode_step(c, 0, q[t], kn[t], vn[t], 0.1, o)
        ms, n = A.arkv_debug_attend_time(c)
        assert n == wl.decode_steps and 0 < ms < 100
        A.arkv_debug_time_attend(c, False)
        buf = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        for pattern in (0, 1, 2):
            us = A.arkv_measure_stream_read(buf, 16 << 20, 20, pattern)
            assert 0 < us < 1e4
    finally:
        A.arkv_cache_destroy(c)
