"""Pins of the end-to-end oracle (Alg. 1) on small trajectories: special cases that
reduce to library attention, brute-force bookkeeping, and the invariants the paper
states (eq. 1 budget, eq. 10 partition, protected window)."""
import numpy as np
import pytest
import torch

from oracle import arkv_oracle as O
from paper_2603_08727_amd import synth


def _prefill(wl, layer=0, b=0):
    k, v, qw = synth.prefill_inputs(wl, layer)
    k, v, qw = (synth.to_numpy_f32(t[b]) for t in (k, v, qw))
    scale = synth.softmax_scale(wl, layer)
    a = O.window_attention(qw, k, scale, wl.group)
    s1, s2 = O.prefill_accumulators(a, wl.group)
    return k, v, a, s1, s2, scale


def _decode(wl, layer=0, b=0):
    q, kn, vn = synth.decode_inputs(wl, layer)
    return tuple(synth.to_numpy_f32(t[:, b]) for t in (q, kn, vn))


def test_below_budget_equals_full_attention():
    """Sec. V-E observation: while the context fits the budget the method is the base model."""
    wl = synth.C1.scaled(prefill=40, budget_frac=3.0, decode_steps=12)      # N = 120 > 52
    k, v, a, s1, s2, scale = _prefill(wl)
    q, kn, vn = _decode(wl)
    cache = O.SequenceCacheOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, bits=4)
    cache.commit(k, v, s1, s2, rho=0.5)
    K, V = k.copy(), v.copy()
    G = wl.group
    for t in range(wl.decode_steps):
        out, fired = cache.decode_step(q[t], kn[t], vn[t], scale)
        assert not fired
        K = np.concatenate([K, kn[t][:, None]], 1); V = np.concatenate([V, vn[t][:, None]], 1)
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.tensor(q[t], dtype=torch.float64)[None, :, None, :],
            torch.tensor(np.repeat(K, G, 0), dtype=torch.float64)[None],
            torch.tensor(np.repeat(V, G, 0), dtype=torch.float64)[None], scale=scale)[0, :, 0].numpy()
        assert np.allclose(out, ref, rtol=1e-10, atol=1e-12)
    assert cache.n_tailors == 0


def test_score_bookkeeping_bruteforce():
    """Every probability row ever produced is stored; s1, s2 and the sample count of each
    surviving token must equal sums over that history (eq. 9 running moments)."""
    wl = synth.C1.scaled(prefill=48, budget_frac=0.5, decode_steps=30, window=4)  # N = 24
    k, v, a, s1, s2, scale = _prefill(wl)
    q, kn, vn = _decode(wl)
    G, W, T = wl.group, wl.window, wl.prefill
    cache = O.SequenceCacheOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, W=W, bits=4)
    hist = [dict() for _ in range(wl.n_kv_heads)]       # per kv-head: pos -> list of samples
    for g in range(wl.n_kv_heads):
        for j in range(T):
            hist[g][j] = [a[g * G + hh, i, j] for hh in range(G) for i in range(W) if T - W + i >= j]
    cache.commit(k, v, s1, s2, rho=0.4)
    assert cache.n_tailors == 1
    for t in range(wl.decode_steps):
        live_before = [set(u.pos.tolist()) | {cache.P + 1} for u in cache.units]
        sum_before = [u.s1.sum() for u in cache.units]
        # replay the attention by hand on the oracle's own dequantised rows
        P = cache.P + 1
        rows = []
        for g, u in enumerate(cache.units):
            keys = np.concatenate([u.kv[:, 0], kn[t][g][None].astype(np.float64)])
            poss = np.append(u.pos, P)
            for hh in range(G):
                lg = scale * keys @ q[t][g * G + hh].astype(np.float64)
                e = np.exp(lg - lg.max()); p = e / e.sum()
                rows.append((g, poss, p))
        n_t = cache.n_tailors
        out, fired = cache.decode_step(q[t], kn[t], vn[t], scale)
        for g, poss, p in rows:
            for pj, pv in zip(poss, p):
                hist[g].setdefault(int(pj), []).append(pv)
        for g, u in enumerate(cache.units):
            if not fired:   # nothing evicted: total mass grew by exactly G
                assert u.s1.sum() == pytest.approx(sum_before[g] + G, rel=1e-12)
            n = O.sample_count(u.pos, cache.P, T, W, G)
            for j, pj in enumerate(u.pos):
                h_ = hist[g][int(pj)]
                assert len(h_) == n[j]
                assert u.s1[j] == pytest.approx(sum(h_), rel=1e-10)
                assert u.s2[j] == pytest.approx(sum(x * x for x in h_), rel=1e-10)
    assert cache.n_tailors > 2


@pytest.mark.parametrize("rho,bits", [(0.5, 4), (0.0, 4), (1.0, 4), (0.3, 2)])
def test_invariants_on_c1(rho, bits):
    """Config 1 run end to end: eq. 1 (bytes within budget), eq. 10 (partition, exact
    survivor count, window Original), monotone states, cadence of the tailor."""
    wl = synth.C1.scaled(bits=bits)
    N, W, d = wl.capacity, wl.window, wl.head_dim
    k, v, a, s1, s2, scale = _prefill(wl)
    q, kn, vn = _decode(wl)
    cache = O.SequenceCacheOracle(wl.n_q_heads, wl.n_kv_heads, d, N, bits=bits)
    cache.commit(k, v, s1, s2, rho=rho)
    n_o, n_q, b = O.budget_counts(rho, N, W)
    assert (n_o, n_q, b) == (cache.n_o, cache.n_q, cache.b) and b == 72
    ever_q = [set() for _ in cache.units]
    steps_since = 0
    for t in range(-1, wl.decode_steps):
        if t >= 0:
            _, fired = cache.decode_step(q[t], kn[t], vn[t], scale)
            steps_since = 0 if fired else steps_since + 1
            assert steps_since <= N - b - W          # slack alpha sets the cadence
        for g, u in enumerate(cache.units):
            live = len(u.pos)
            assert live <= N - 1 and len(set(u.pos.tolist())) == live
            no, nq = cache.counts(g)
            assert no + nq == live and set(u.state.tolist()) <= {O.STATE_O, O.STATE_Q}
            assert cache.live_bytes(g) <= N * 4 * d                      # eq. 1 per kv-head
            win = u.pos > cache.P - W
            assert win.sum() == W and (u.state[win] == O.STATE_O).all()
            assert nq <= b and no <= n_o + W + (N - b - W)
            if rho == 1.0:
                assert nq == 0
            if rho == 0.0 and t == -1:
                assert no == W
            qs = set(u.pos[u.state == O.STATE_Q].tolist())
            assert not (ever_q[g] & set(u.pos[u.state == O.STATE_O].tolist()))   # never promoted
            ever_q[g] |= qs
            for pj in qs:                       # stored codes reproduce the value attention sees
                e = u.q[pj]; j = int(np.nonzero(u.pos == pj)[0][0])
                assert np.array_equal(u.kv[j, 0], O.dequantize_row(e["k_codes"], e["k_scale"], e["k_zero"]))
                assert np.array_equal(u.kv[j, 1], O.dequantize_row(e["v_codes"], e["v_scale"], e["v_zero"]))
                # both rows went through the quantiser of the bf16 row (K and V alike)
                for r, nm in ((0, "k"), (1, "v")):
                    c, sc, zr = O.quantize_row(u.raw[j, r], bits)
                    assert np.array_equal(c, e[nm + "_codes"]) and np.array_equal(sc, e[nm + "_scale"])
                    assert np.array_equal(zr, e[nm + "_zero"])
        if t == -1:
            assert all(len(u.pos) == b + W for u in cache.units)
    assert cache.n_tailors == 1 + (wl.decode_steps // (N - b - W))


def test_lockstep_override_is_used():
    """With scores supplied from outside, the selection follows them exactly."""
    wl = synth.C1.scaled(prefill=64, budget_frac=0.5, window=4)      # N = 32
    k, v, a, s1, s2, scale = _prefill(wl)
    cache = O.SequenceCacheOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, W=4, bits=4)
    T = wl.prefill
    over = [{j: np.float32(j % 7) for j in range(T)} for _ in range(wl.n_kv_heads)]
    cache.commit(k, v, s1, s2, rho=0.5, S_override=over)
    n_o, n_q, b = O.budget_counts(0.5, 32, 4)
    order = sorted(range(T - 4), key=lambda j: (-(j % 7), j))
    for u in cache.units:
        keep = set(order[:b]) | set(range(T - 4, T))
        assert set(u.pos.tolist()) == keep
        assert set(u.pos[u.state == O.STATE_O].tolist()) == set(order[:n_o]) | set(range(T - 4, T))


@pytest.mark.parametrize("delta", [-1, 0, 1])
def test_prompt_that_exactly_fills_the_cache(delta):
    """T = N - 1: the prompt fits and nothing is removed until the first decode step fills the cache; T = N and
    T = N + 1: the first tailor runs at commit, so that the first append has room (Sec. IV-F: the tailor is
    triggered when the cache reaches the limit)."""
    wl = synth.C1.scaled(name="exact", prefill=128 + delta, budget_frac=1.0, decode_steps=2)
    N, W = 128, wl.window
    k, v, a, s1, s2, scale = _prefill(wl)
    cache = O.SequenceCacheOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, N)
    cache.commit(k, v, s1, s2, rho=0.5)
    b = O.budget_counts(0.5, N, W)[2]
    if delta < 0:
        assert cache.n_tailors == 0 and all(len(u.pos) == N - 1 for u in cache.units)
    else:
        assert cache.n_tailors == 1 and all(len(u.pos) == b + W for u in cache.units)
    q, kn, vn = _decode(wl)
    _, fired = cache.decode_step(q[0], kn[0], vn[0], scale)
    assert fired == (delta < 0)                 # N - 1 + 1 = N live tokens: now it is full
    assert all(len(u.pos) <= N - 1 for u in cache.units)


@pytest.mark.parametrize("rho,bits,window", [(0.4, 4, 32), (0.0, 2, 8), (1.0, 4, 16), (0.6, 8, 32)])
def test_every_step_reading_trajectory(rho, bits, window):
    """Sec. IV-F first sentence read literally ("at each step"): no slack, the cache stays full.  What that
    reading fixes without running anything: after the commit and after every decode step a kv-head holds N - 1
    tokens; every step runs one tailor (n_tailors = 1 + steps); each tailor of a decode step evicts exactly one
    token per kv-head, and that token is the one a full sort of the eligible tokens by (score descending,
    position ascending) puts last; the window stays Original; eq. 1 holds."""
    d = 128 if bits == 8 else 64
    wl = synth.C1.scaled(name="every", prefill=200, budget_frac=0.3, decode_steps=20, window=window, bits=bits,
                         head_dim=d)
    N, W = wl.capacity, wl.window
    k, v, a, s1, s2, scale = _prefill(wl)
    q, kn, vn = _decode(wl)
    cache = O.SequenceCacheOracle(wl.n_q_heads, wl.n_kv_heads, d, N, W=W, bits=bits, every_step=True)
    cache.commit(k, v, s1, s2, rho=rho)
    assert cache.b == N - W - 1 and cache.n_o == min(int(np.floor(rho * (N - W))), N - W - 1)
    assert cache.n_tailors == 1 and all(len(u.pos) == N - 1 for u in cache.units)
    for t in range(wl.decode_steps):
        before = [set(u.pos.tolist()) for u in cache.units]
        # scores the tailor of this step will rank on, replayed by hand from the cache's own rows
        P = cache.P + 1
        last = []
        for g, u in enumerate(cache.units):
            keys = np.concatenate([u.kv[:, 0], kn[t][g][None].astype(np.float64)])
            poss = np.append(u.pos, P)
            c1 = np.append(u.s1, 0.0); c2 = np.append(u.s2, 0.0)
            for hh in range(wl.group):
                lg = scale * keys @ q[t][g * wl.group + hh].astype(np.float64)
                e = np.exp(lg - lg.max()); p = e / e.sum()
                c1 += p; c2 += p * p
            n = wl.group * (P - np.maximum(poss, wl.prefill - W) + 1)
            mu = c1 / n
            S = mu + cache.gamma * np.maximum(c2 / n - mu * mu, 0.0)
            el = poss < P + 1 - W
            ranked = sorted(zip(-S[el], poss[el]))                  # score descending, position ascending
            last.append(int(ranked[-1][1]))
        _, fired = cache.decode_step(q[t], kn[t], vn[t], scale)
        assert fired and cache.n_tailors == 2 + t
        for g, u in enumerate(cache.units):
            now = set(u.pos.tolist())
            assert len(u.pos) == N - 1
            gone = (before[g] | {P}) - now
            assert gone == {last[g]}                                # one eviction, the lowest-ranked eligible token
            win = u.pos > cache.P - W
            assert win.sum() == W and (u.state[win] == O.STATE_O).all()
            no, nq = cache.counts(g)
            assert no + nq == N - 1 and no <= cache.n_o + W
            if rho == 1.0:
                assert nq == 0
            assert cache.live_bytes(g) <= N * 4 * d
