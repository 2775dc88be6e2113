"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (one
arkv_decode_step per layer, the configuration's whole batch): prompt scoring, commit with the first
tailor, and a few decode steps of ONE layer of configurations 2, 3 and 4, every unit compared with
the oracle (states, codes, scales bit-exact; outputs, scores, statistics at 2e-3)."""
import numpy as np
import pytest

from paper_2603_08727_amd import synth
from helpers import SideBySide

pytestmark = pytest.mark.gpu


def _run(wl, steps):
    sb = SideBySide(wl)
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


@pytest.mark.parametrize("rho", [None, 0.5])
def test_c3_full_size_decode_time_tailor(rho):
    """Config 3's shape with almost no slack (alpha = 0.99: b = 8078 of N = 8192, a tailor every 82 decode steps) so
    that a decode-time tailor over the full-size cache (eq. 10 on 8.2K tokens per unit, 32 units: select,
    demotion with in-place quantisation, compaction) is compared with the oracle, then a few steps more.  rho = 0.5 forces a mixed cache, so that
    rows are demoted and quantised in place; None takes the scored ratio of this layer."""
    wl = synth.C3.scaled(name="c3_tight", n_layers=1, alpha=0.99)
    sb = SideBySide(wl, rho_override=rho)
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
