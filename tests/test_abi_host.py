"""CPU-side checks of the C-ABI library: it loads, exports what include/arkv.h declares, rejects bad
arguments before touching a GPU, and its host-only entry points agree with the oracle."""
import os
import re

import numpy as np
import pytest

from oracle import arkv_oracle as O
from paper_2603_08727_amd import binding as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "arkv.h")).read()
    declared = set(re.findall(r"\b(arkv_[a-z0-9_]+)\s*\(", hdr))
    assert declared, "no declarations found"
    lib = A.load()
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in arkv.h but not exported"
    assert declared == set(A.EXPORTED)


def test_measurement_library_exports_what_its_header_declares_and_is_not_in_the_product():
    hdr = open(os.path.join(ROOT, "include", "arkv_measure.h")).read()
    declared = set(re.findall(r"\b(arkv_measure_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(A.MEASURE_EXPORTED)
    mlib = A.load_measure()
    for name in declared:
        assert hasattr(mlib, name), f"{name} declared in arkv_measure.h but not exported"
        assert not hasattr(A.load(), name), f"{name} must not be part of libarkv.so"
    import ctypes as C
    us = C.c_float()
    assert mlib.arkv_measure_stream_read(None, 0, 0, 1, 0, None, C.byref(us)) == -1      # argument check, no GPU


def test_phase_trace_hook_is_off_in_the_product_build():
    import ctypes as C
    buf = (C.c_uint64 * 8)()
    lib = A.load()
    assert lib.arkv_debug_phase_trace(0, buf, 1) == A.EUNSUPPORTED
    assert lib.arkv_debug_phase_trace(3, buf, 1) == A.EINVAL and lib.arkv_debug_phase_trace(0, None, 1) == A.EINVAL
    assert lib.arkv_debug_phase_trace(0, buf, 0) == A.EINVAL and lib.arkv_debug_phase_trace(0, buf, 8193) == A.EINVAL


def test_strerror_and_defaults():
    assert A.strerror(0) == "ok" and "invalid" in A.strerror(A.EINVAL)
    cfg = A.arkv_config_default()
    assert cfg.window == 32 and cfg.alpha == 0.75 and cfg.quant_bits == 4 and cfg.group_size == 32
    assert [round(x, 3) for x in cfg.tau] == [7.774, 5.407, 5.528] and round(cfg.gamma, 2) == 263.81


def _cfg(**kw):
    base = dict(n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2, head_dim=64, capacity_tokens=128)
    base.update(kw)
    return A.arkv_config_default(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(n_layers=0), A.EINVAL), (dict(n_q_heads=7), A.EINVAL), (dict(window=127), A.EINVAL),
    (dict(alpha=0.0), A.EINVAL), (dict(alpha=1.5), A.EINVAL), (dict(gamma=-1.0), A.EINVAL),
    (dict(group_size=64), A.EINVAL), (dict(head_dim=96), A.EUNSUPPORTED),
    (dict(quant_bits=3), A.EUNSUPPORTED), (dict(n_q_heads=6, n_kv_heads=2), A.EUNSUPPORTED),
    (dict(tau=(1.0, 0.0, 1.0)), A.EINVAL), (dict(tailor_policy=2), A.EINVAL), (dict(budget_mode=3), A.EINVAL),
    (dict(capacity_tokens=1 << 20), A.EUNSUPPORTED),
])
def test_create_rejects_bad_config_without_gpu(kw, code):
    with pytest.raises(A.ArkvError) as e:
        A.arkv_cache_create(_cfg(**kw))
    assert e.value.code == code


def test_null_handles_are_errors_not_crashes():
    lib = A.load()
    assert lib.arkv_cache_destroy(None) == A.OK
    assert lib.arkv_decode_step(None, 0, None, None, None, 1.0, None, None) == A.EINVAL
    assert lib.arkv_prefill_stats(None, 0, None, None, 10, 1.0, None, None) == A.EINVAL
    assert lib.arkv_cache_create(None, None) == A.EINVAL


@pytest.mark.parametrize("N,W,alpha", [(128, 32, 0.75), (2048, 32, 0.75), (8192, 32, 0.75), (16384, 32, 0.75),
                                       (40, 8, 0.5), (100, 4, 1.0), (64, 16, 0.9)])
def test_budget_counts_match_oracle(N, W, alpha):
    cfg = _cfg(capacity_tokens=N, window=W, alpha=alpha)
    for rho in np.linspace(0, 1, 41, dtype=np.float32):
        got = A.arkv_budget_counts(cfg, float(rho))
        want = O.budget_counts(float(rho), N, W, float(np.float32(alpha)))
        assert got == want
    cfgb = _cfg(capacity_tokens=N, window=W, alpha=alpha, budget_mode=1, head_dim=128, quant_bits=4)
    for rho in (0.0, 0.25, 0.9, 1.0):
        assert A.arkv_budget_counts(cfgb, rho) == O.budget_counts(rho, N, W, float(np.float32(alpha)),
                                                                  byte_costs=O.row_bytes(128, 4))
    cfg1 = _cfg(capacity_tokens=N, window=W, alpha=alpha, tailor_policy=1)
    for rho in (0.0, 0.3, 1.0):
        assert A.arkv_budget_counts(cfg1, rho) == O.budget_counts(rho, N, W, float(np.float32(alpha)), every_step=True)
        assert A.arkv_budget_counts(cfg1, rho)[2] == N - W - 1


def test_oq_ratio_matches_oracle():
    rng = np.random.default_rng(0)
    L, B = 7, 3
    stats = np.stack([rng.uniform(3, 9, (L, B)), 10 ** rng.uniform(-9, -5, (L, B)), rng.uniform(3, 500, (L, B))],
                     axis=-1).astype(np.float32)
    stats[2, 1] = (5.0, 0.0, 0.0)            # a uniform layer: q = 0
    stats[:, 2] = (np.log(100.0), 0.0, 0.0)  # a sequence where every layer is uniform: all rho = 1
    tau = np.float32(O.PAPER_TAU)
    rho = A.arkv_oq_ratio(stats, tau)
    for b in range(B):
        q = [O.oq_score(*stats[l, b].astype(np.float64), tau=tau.astype(np.float64)) for l in range(L)]
        assert np.allclose(rho[:, b], O.oq_ratio(q), rtol=1e-6)
    assert (rho[:, 2] == 1).all() and rho[2, 1] == 0 and rho.max() == 1
    bad = stats.copy(); bad[0, 0, 1] = np.nan
    with pytest.raises(A.ArkvError):
        A.arkv_oq_ratio(bad, tau)


def test_split_ranges_partition_the_pools():
    """Host logic of the split-K decomposition: for any counts the splits' row ranges are contiguous, ordered,
    cover both pools exactly once, and carry about equal weight (a packed row weighs w/16 of a bf16 row; the
    last split is charged 32 rows for the appended token; packed rows are dealt in blocks of 32)."""
    rng = np.random.default_rng(1)
    cases = [(0, 0, 14, 1), (1, 0, 14, 1), (0, 5, 14, 4), (6180, 0, 14, 16), (60, 6120, 14, 16), (4140, 2040, 14, 16),
             (8209, 19584, 16, 128), (33, 1, 1, 7)]
    cases += [(int(rng.integers(0, 9000)), int(rng.integers(0, 20000)), int(rng.integers(1, 17)), int(rng.integers(1, 129)))
              for _ in range(40)]
    for cO, cQ, w, S in cases:
        ends_o, ends_q, weights = 0, 0, []
        for s in range(S):
            ao, bo, aq, bq = A.arkv_debug_split_range(cO, cQ, w, S, s)
            assert ao == ends_o and aq == ends_q and ao <= bo <= cO and aq <= bq <= cQ, (cO, cQ, w, S, s)
            ends_o, ends_q = bo, bq
            weights.append(16 * (bo - ao) + w * (bq - aq) + (16 * 32 if s == S - 1 else 0))
            assert (aq % 32 == 0 or aq == bq == cQ) and (bq % 32 == 0 or bq == cQ)   # packed rows are dealt in whole value blocks
        assert ends_o == cO and ends_q == cQ
        assert max(weights) - min(weights) <= 2 * 16 + 16 * 32 + 2 * 32 * w, (cO, cQ, w, S, weights)
    for bad in [(-1, 0, 14, 4, 0), (0, 0, 0, 4, 0), (0, 0, 14, 0, 0), (0, 0, 14, 129, 0), (0, 0, 14, 4, 4)]:
        with pytest.raises(A.ArkvError):
            A.arkv_debug_split_range(*bad)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; --gpus N > 1 exits with a message before anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_product_path_does_not_import_the_oracle():
    """The oracle is test infrastructure: nothing under the package or in the binding's import chain may load it."""
    import os
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2603_08727_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "arkv_oracle" not in text, f
