"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (one
arkv_decode_step per layer, the configuration's whole batch): prompt scoring, commit with the first
tailor, and a few decode steps of ONE layer of configurations 2, 3 and 4, every unit compared with
the oracle (states, codes, scales bit-exact; outputs, scores, statistics at 2e-3)."""
import numpy as np
import pytest

from paper_2603_08727_amd import synth
from helpers import SideBySide

pytestmark = pytest.mark.gpu


def _run(wl, steps, lockstep=True):
    sb = SideBySide(wl, lockstep=lockstep)
    try:
        sb.prefill()
        sb.commit()
        sb.decode(steps, check_every=steps)
        print(wl.name, {k: f"{v:.2e}" for k, v in sb.max_err.items()}, flush=True)
        sb.assert_within_tol()
        for oc in sb.oracles.values():
            assert oc.n_tailors == 1
            for g in range(wl.n_kv_heads):
                assert len(oc.units[g].pos) == oc.b + wl.window + steps
    finally:
        sb.close()


def test_c2_llama3_8k_one_layer():
    _run(synth.C2.scaled(n_layers=1), steps=4)


def test_c3_qwen3_32k_batch4_one_layer():
    _run(synth.C3.scaled(n_layers=1), steps=3)


def test_c4_128k_2bit_one_layer():
    _run(synth.C4.scaled(n_layers=1), steps=3)


def test_c3_qwen3_32k_batch4_one_layer_free_running():
    """The same layer without the score hand-over: the first tailor ranks 32736 prompt tokens per kv-head on each
    side's own scores; choices are compared under the score-band rule (2e-3 around the two cuts)."""
    _run(synth.C3.scaled(n_layers=1), steps=3, lockstep=False)


def test_c4_128k_2bit_one_layer_free_running():
    """The 128K-context configuration without the score hand-over: 131040 prompt tokens per kv-head ranked on each
    side's own scores, 2-bit rows."""
    _run(synth.C4.scaled(n_layers=1), steps=3, lockstep=False)


def test_c2_llama3_8k_one_layer_free_running():
    _run(synth.C2.scaled(n_layers=1), steps=4, lockstep=False)


@pytest.mark.parametrize("rho,lockstep", [(None, True), (0.5, True), (0.5, False)])
def test_c3_full_size_decode_time_tailor(rho, lockstep):
    """Config 3's shape with almost no slack (alpha = 0.99: b = 8078 of N = 8192, a tailor every 82 decode steps) so
    that a decode-time tailor over the full-size cache (eq. 10 on 8.2K tokens per unit, 32 units: select,
    demotion with in-place quantisation, compaction) is compared with the oracle, then a few steps more.  rho = 0.5 forces a mixed cache, so that
    rows are demoted and quantised in place; None takes the scored ratio of this layer.  lockstep False: no score
    hand-over, both tailors compared under the score-band rule."""
    wl = synth.C3.scaled(name="c3_tight", n_layers=1, alpha=0.99)
    sb = SideBySide(wl, rho_override=rho, lockstep=lockstep)
    try:
        sb.prefill()
        sb.commit()
        steps = wl.capacity - int(wl.alpha * (wl.capacity - wl.window)) - wl.window + 6
        sb.decode(steps, check_every=steps)
        print(wl.name, steps, {k: f"{v:.2e}" for k, v in sb.max_err.items()}, flush=True)
        sb.assert_within_tol()
        for oc in sb.oracles.values():
            assert oc.n_tailors == 2
            if rho is not None:
                assert all(oc.counts(g)[1] > 1000 for g in range(wl.n_kv_heads))     # Quantized tokens per unit
    finally:
        sb.close()


def _run_scorer(wl):
    sb = SideBySide(wl)
    try:
        sb.prefill()
        sb.commit()          # compares the survivors' window sums (s1, s2), states and rows as well
        print(wl.name, {k: f"{v:.2e}" for k, v in sb.max_err.items()}, flush=True)
        sb.assert_within_tol()
    finally:
        sb.close()


def test_c5_prefill_scorer_16k_batch8_one_layer():
    """The prefill-scorer stress shape (16K context, batch 8, sharp and flat heads), one layer, paper window."""
    _run_scorer(synth.C5.scaled(n_layers=1))


def test_c5_prefill_scorer_window_128():
    """Same shape with a 4x observation window (512 query rows per unit), two sequences."""
    _run_scorer(synth.C5.scaled(n_layers=1, batch=2, window=128))


@pytest.mark.parametrize("window,hq,hkv", [(64, 32, 8), (16, 32, 8), (64, 16, 8), (128, 16, 8), (32, 64, 8)])
def test_prefill_scorer_row_tile_counts(window, hq, hkv):
    """Every number of 32-row tiles the scorer instantiates (2, 4, 8, 16; 4 and 8 waves per workgroup) on a prompt
    long enough for several unmasked key tiles per wave, one sequence."""
    _run_scorer(synth.C5.scaled(name=f"scorer_w{window}_g{hq // hkv}", n_layers=1, batch=1, window=window,
                                n_q_heads=hq, n_kv_heads=hkv, prefill=4096 + 77))


def test_c3_natural_tailor_cadence_invariants():
    """Config 3 at full size, two layers, stepped past the first decode-time tailor at its natural cadence
    (N - b - W = 2040 steps) without the oracle: what must hold at any size.  Every unit holds b + W + (steps since
    the tailor) tokens; positions are distinct, the window and every token generated since the tailor are there and
    Original; Original counts respect the budget; scores are finite and non-negative; live bytes within eq. 1."""
    import torch
    from paper_2603_08727_amd import binding as A
    from helpers import make_cfg
    wl = synth.C3.scaled(name="c3_cadence", n_layers=2)
    cfg = make_cfg(wl)
    L, B, Hq, Hkv, d, T, W, N = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.prefill, wl.window, wl.capacity
    U = B * Hkv
    cache = A.arkv_cache_create(cfg)
    try:
        scales = [synth.softmax_scale(wl, l) for l in range(L)]
        stats = torch.zeros((L, B, 3), dtype=torch.float32, device="cuda")
        for l in range(L):
            k, v, qw = synth.prefill_inputs(wl, l, device="cuda")
            A.arkv_prefill_stats(cache, l, qw, k, T, scales[l], stats[l])
        rho = A.arkv_oq_ratio(stats.cpu().numpy(), wl.tau)
        rho[1, :] = 0.5                                    # layer 1: a mixed cache whatever the scorer says
        for l in range(L):
            k, v, qw = synth.prefill_inputs(wl, l, device="cuda")
            A.arkv_prefill_commit(cache, l, k, v, T, rho[l])
        b = int(np.floor(np.float32(wl.alpha) * (N - W)))
        steps = (N - b - W) + 25
        dq = [synth.decode_inputs(wl, l, steps, device="cuda") for l in range(L)]
        out = torch.empty((B, Hq, d), dtype=torch.bfloat16, device="cuda")
        for t in range(steps):
            for l in range(L):
                A.arkv_decode_step(cache, l, dq[l][0][t], dq[l][1][t], dq[l][2][t], scales[l], out)
        torch.cuda.synchronize()
        assert torch.isfinite(out.float()).all()
        since = steps - (N - b - W)                         # steps after the tailor fired
        for l in range(L):
            n_tailors = A.arkv_cache_progress(cache, l)[0]
            assert n_tailors == 2                           # the one at commit and the one at the cadence
            ex = A.arkv_cache_export(cache, l, cfg, rows=False, codes=False)
            no, nq, ne, lb = A.arkv_cache_counters(cache, l, U)
            n_o_target = [A.arkv_budget_counts(cfg, float(rho[l, s]))[0] for s in range(B)]
            for u in range(U):
                n = int(ex["n_live"][u])
                assert n == b + W + since == no[u] + nq[u]
                pos = ex["pos"][u, :n]; st = ex["state"][u, :n]
                assert len(np.unique(pos)) == n and pos.min() >= 0 and pos.max() == T + steps - 1
                recent = pos >= T + steps - (W + since)      # the window at the tailor plus everything since
                assert recent.sum() == W + since and (st[recent] == 0).all()
                assert no[u] - (W + since) <= n_o_target[u // Hkv]
                assert ne[u] == T + steps - n
                s1 = ex["s1"][u, :n]; s2 = ex["s2"][u, :n]
                assert np.isfinite(s1).all() and np.isfinite(s2).all() and (s1 >= 0).all() and (s2 >= 0).all()
                assert lb[u] <= N * 4 * d
            if l == 1:
                assert (nq > 1000).all()
    finally:
        A.arkv_cache_destroy(cache)


def test_c4_shape_whole_prompt_kept():
    """The largest cache of the benchmark: configuration 4's 131072-token prompt with a limit above its length,
    so every token stays Original (131K rows per unit, 32 splits of 4K rows each); three decode steps, every unit's
    outputs, scores and rows against the oracle."""
    T = synth.C4.prefill
    wl = synth.C4.scaled(name="c4_full_cache", n_layers=1, budget_frac=(T + 64) / T, decode_steps=3)
    sb = SideBySide(wl)
    try:
        sb.prefill()
        sb.commit()
        sb.decode(3, check_every=3)
        print(wl.name, {k: f"{v:.2e}" for k, v in sb.max_err.items()}, flush=True)
        sb.assert_within_tol()
        for oc in sb.oracles.values():
            assert oc.n_tailors == 0 and all(len(u.pos) == T + 3 for u in oc.units)
    finally:
        sb.close()


@pytest.mark.parametrize("rho", [None, 0.5])
def test_c3_full_size_tailor_at_every_step(rho):
    """Config 3's shape under tailor_policy 1 (no slack: the cache stays full, one token leaves per unit and
    step): commit plus four decode steps, each followed by a tailor over 8160 eligible tokens per unit."""
    wl = synth.C3.scaled(name="c3_every_step", n_layers=1, decode_steps=4)
    sb = SideBySide(wl, rho_override=rho, every_step=True)
    try:
        sb.prefill()
        sb.commit()
        sb.decode(4, check_every=1)
        print(wl.name, rho, {k: f"{v:.2e}" for k, v in sb.max_err.items()}, flush=True)
        sb.assert_within_tol()
        for oc in sb.oracles.values():
            assert oc.n_tailors == 5 and all(len(u.pos) == wl.capacity - 1 for u in oc.units)
    finally:
        sb.close()


def test_c3_full_size_fp8_rows_byte_budget_decode_time_tailor():
    """The paper's own Quantized format (fp8 codes, one scale per row) under the byte reading of the budget
    (eq. 1, eq. 8), at config 3's size with a mixed cache: commit, the steps up to the first decode-time tailor
    and a few more; live bytes stay within the limit on both sides."""
    wl = synth.C3.scaled(name="c3_fp8_bytes", n_layers=1, alpha=0.99, bits=8)
    sb = SideBySide(wl, rho_override=0.5, byte_budget=True)
    try:
        sb.prefill()
        sb.commit()
        steps = wl.capacity - int(wl.alpha * (wl.capacity - wl.window)) - wl.window + 6
        sb.decode(steps, check_every=steps)
        print(wl.name, steps, {k: f"{v:.2e}" for k, v in sb.max_err.items()}, flush=True)
        sb.assert_within_tol()
        for oc in sb.oracles.values():
            assert oc.n_tailors == 2
            for g in range(wl.n_kv_heads):
                assert oc.counts(g)[1] > 1000
                assert oc.live_bytes(g) <= wl.capacity * 4 * wl.head_dim
    finally:
        sb.close()
