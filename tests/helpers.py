"""Shared plumbing of the GPU parity tests: runs the HIP path (through the C ABI binding) and the
CPU oracle side by side on the same synthetic inputs and compares them."""
from __future__ import annotations

import copy

import numpy as np
import torch

from oracle import arkv_oracle as O
from paper_2603_08727_amd import binding as A
from paper_2603_08727_amd import synth

TOL = 2e-3                  # attention outputs, scores, statistics (fp32 accumulation)


def rel_err(x, ref):
    """max |x - ref| / max |ref| over one tensor (element-wise relative error is meaningless for
    values that cancel to ~0)."""
    x = np.asarray(x, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    return float(np.abs(x - ref).max() / den) if den > 0 else float(np.abs(x).max())


def bf16_round(x32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bits, round to nearest even (for checking the library's final rounding)."""
    u = np.asarray(x32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def score_band_check(S, pos, state_ref, state_got, n_o, b, tol=TOL, where=None):
    """The free-running rule for one tailor of one kv-head.  S, pos: the reference's scores and positions of the
    eligible tokens; state_ref / state_got: the state each side gave them.  The two may differ only for tokens
    whose score lies within tol (relative) of the score at one of the two cuts of eq. 10: rank n_o (Original /
    Quantized) and rank b (kept / evicted); the tokens on either side of a cut define it.  Raises AssertionError
    for a difference outside the band; returns True when there is no difference at all."""
    S = np.asarray(S, dtype=np.float64)
    bad = np.nonzero(np.asarray(state_got) != np.asarray(state_ref))[0]
    if not len(bad):
        return True
    ranked = np.sort(S)[::-1]
    cuts = [ranked[r] for r in (n_o - 1, n_o, b - 1, b) if 0 <= r < len(ranked)]
    for j in bad:
        near = min((abs(S[j] - c) / abs(c) if c != 0 else abs(S[j])) for c in cuts)
        assert near <= tol, ("a token outside the score band changed state", where, int(np.asarray(pos)[j]),
                             float(S[j]), cuts, int(state_got[j]), int(state_ref[j]))
    return False


def make_cfg(wl: synth.Workload, every_step=False, byte_budget=False):
    return A.arkv_config_default(
        n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
        head_dim=wl.head_dim, capacity_tokens=wl.capacity, window=wl.window, alpha=wl.alpha,
        gamma=wl.gamma, tau=wl.tau, quant_bits=wl.bits, tailor_policy=1 if every_step else 0,
        budget_mode=1 if byte_budget else 0)


class SideBySide:
    """One workload on both sides.  Scores the prompt, commits, then steps in lock-step: whenever the
    GPU ran a tailor, the oracle's tailor of the same step ranks on the GPU's fp32 scores, so that
    states / codes / scales can be compared bit for bit; everything floating point is compared at TOL.
    lockstep=False is the free-running protocol: the oracle ranks on its own fp64 scores, every tailor's
    choice is compared under the score-band rule (score_band_check), and where the two sides split near-tied
    tokens differently the oracle goes on from the GPU's choice so that the comparison can continue."""

    def __init__(self, wl: synth.Workload, rho_override=None, device="cuda", every_step=False, lockstep=True,
                 byte_budget=False, mutate_prefill=None, mutate_decode=None):
        # mutate_prefill(layer, k, v, qw) / mutate_decode(layer, q, k_new, v_new): in-place edits of the drawn
        # CPU tensors before either side sees them (degenerate rows, zero queries, ...)
        self.mutate_prefill, self.mutate_decode = mutate_prefill, mutate_decode
        self.wl = wl
        self.dev = device
        self.every_step = every_step
        self.lockstep = lockstep       # False: the oracle ranks on its own fp64 scores (free-running protocol)
        self.byte_budget = byte_budget
        self.cfg = make_cfg(wl, every_step, byte_budget)
        self.cache = A.arkv_cache_create(self.cfg)
        self.U = wl.batch * wl.n_kv_heads
        self.rho_override = rho_override
        self.oracles = {}        # (layer, b) -> SequenceCacheOracle
        self.scales = [synth.softmax_scale(wl, l) for l in range(wl.n_layers)]
        self.stats_gpu = None
        self.stats_ref = None
        self.max_err = dict(out=0.0, s1=0.0, s2=0.0, S=0.0, stats=0.0)
        self.band_tailors = 0          # free-running tailors compared under the score-band rule
        self.band_divergences = 0      # ... of which the two sides chose differently (inside the band)

    def close(self):
        A.arkv_cache_destroy(self.cache)

    # ---- prefill ---------------------------------------------------------------------------------
    def prefill(self):
        wl = self.wl
        L, B = wl.n_layers, wl.batch
        stats = torch.zeros((L, B, 3), dtype=torch.float32, device=self.dev)
        self.inputs = []
        ref_stats = np.zeros((L, B, 3))
        ref_acc = {}
        for l in range(L):
            k, v, qw = synth.prefill_inputs(wl, l)          # CPU draw, copied to the GPU
            if self.mutate_prefill is not None:
                self.mutate_prefill(l, k, v, qw)
            self.inputs.append((k, v, qw))
            kd, qd = k.to(self.dev), qw.to(self.dev)
            A.arkv_prefill_stats(self.cache, l, qd, kd, wl.prefill, self.scales[l], stats[l])
            for b in range(B):
                a = O.window_attention(synth.to_numpy_f32(qw[b]), synth.to_numpy_f32(k[b]), self.scales[l], wl.group)
                H, V, K, _ = O.layer_statistics(a, wl.window)
                ref_stats[l, b] = (H, V, K)
                ref_acc[(l, b)] = O.prefill_accumulators(a, wl.group)
        torch.cuda.synchronize()
        self.stats_gpu = stats.cpu().numpy()
        self.stats_ref = ref_stats
        err = np.abs(self.stats_gpu - ref_stats) / np.maximum(np.abs(ref_stats), 1e-300)
        self.max_err["stats"] = float(err.max())
        # OQ ratio: the library's host routine on the GPU statistics, the oracle's on its own
        self.rho_gpu = A.arkv_oq_ratio(self.stats_gpu, wl.tau)
        q = np.array([[O.oq_score(*ref_stats[l, b], tau=wl.tau) for b in range(B)] for l in range(L)])
        self.rho_ref = np.stack([O.oq_ratio(q[:, b]) for b in range(B)], axis=1)
        self.ref_acc = ref_acc

    def commit(self):
        wl = self.wl
        for l in range(wl.n_layers):
            k, v, _ = self.inputs[l]
            rho = self.rho_gpu[l] if self.rho_override is None else np.full(wl.batch, self.rho_override, np.float32)
            A.arkv_prefill_commit(self.cache, l, k.to(self.dev), v.to(self.dev), wl.prefill, rho)
            over = self._gpu_scores(l) if wl.prefill >= wl.capacity else None
            for b in range(wl.batch):
                oc = O.SequenceCacheOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, W=wl.window,
                                           alpha=float(np.float32(wl.alpha)), gamma=float(np.float32(wl.gamma)),
                                           bits=wl.bits, every_step=self.every_step, byte_budget=self.byte_budget)
                s1, s2 = self.ref_acc[(l, b)]
                if over is not None:
                    self._check_scores(oc, l, b, over, commit=(s1, s2))
                args = (synth.to_numpy_f32(k[b]), synth.to_numpy_f32(v[b]), s1, s2, float(rho[b]))
                mine = None if over is None else over[b * wl.n_kv_heads:(b + 1) * wl.n_kv_heads]
                oc.commit(*args, S_override=mine if self.lockstep else None)
                if over is not None and not self.lockstep and not self._same_choice_or_in_band(oc, l, b):
                    # the two sides split near-tied tokens differently (allowed): go on from the GPU's choice
                    oc = O.SequenceCacheOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, W=wl.window,
                                               alpha=float(np.float32(wl.alpha)), gamma=float(np.float32(wl.gamma)),
                                               bits=wl.bits, every_step=self.every_step, byte_budget=self.byte_budget)
                    oc.commit(*args, S_override=mine)
                self.oracles[(l, b)] = oc
            self.compare_state(l)

    def _gpu_scores(self, layer):
        """Per unit: dict position -> fp32 score of the tailor the GPU just ran."""
        mt = max(self.wl.prefill, 4 * self.wl.capacity + 64)
        cnt, pos, sc = A.arkv_debug_last_tailor_scores(self.cache, layer, self.U, mt)
        assert (cnt >= 0).all()
        return [dict(zip(pos[u, :cnt[u]].tolist(), sc[u, :cnt[u]])) for u in range(self.U)]

    def _check_scores(self, oc, l, b, over, commit=None):
        """GPU scores vs the oracle's own fp64 scores of the same eligible tokens (TOL)."""
        wl = self.wl
        for g in range(wl.n_kv_heads):
            d = over[b * wl.n_kv_heads + g]
            if commit is not None:
                T = wl.prefill
                posr = np.arange(T - wl.window)
                n = O.sample_count(posr, T - 1, T, wl.window, wl.group)
                Sref = O.hh_score(commit[0][g][:T - wl.window], commit[1][g][:T - wl.window], n, oc.gamma)
            else:
                u = oc.units[g]
                el = u.pos < oc.P + 1 - wl.window
                posr = u.pos[el]
                Sref = oc.scores(g)[el]
            assert set(d.keys()) == set(posr.tolist())
            Sg = np.array([d[int(p)] for p in posr])
            assert (Sg >= 0).all()
            self.max_err["S"] = max(self.max_err["S"], rel_err(Sg, Sref))

    def _same_choice_or_in_band(self, oc, layer, b):
        """Free-running protocol: the oracle has just tailored on its OWN fp64 scores; the GPU ranked the same
        tokens on its fp32 scores.  Applies score_band_check per kv-head; True when both sides chose alike."""
        wl = self.wl
        ex = A.arkv_cache_export(self.cache, layer, self.cfg)
        self.band_tailors += 1
        same = True
        for g in range(wl.n_kv_heads):
            u = b * wl.n_kv_heads + g
            lt = oc.last_tailor[g]
            n = ex["n_live"][u]
            gpu_state = dict(zip(ex["pos"][u, :n].tolist(), ex["state"][u, :n].tolist()))
            got = np.array([gpu_state.get(int(p), O.STATE_E) for p in lt["pos"]])
            same &= score_band_check(lt["S"], lt["pos"], lt["new_state"], got, oc.n_o, oc.b, where=(layer, u))
        if not same:
            self.band_divergences += 1
        return same

    # ---- decode ----------------------------------------------------------------------------------
    def decode(self, steps=None, check_every=1):
        wl = self.wl
        S = wl.decode_steps if steps is None else steps
        ins = [synth.decode_inputs(wl, l, S) for l in range(wl.n_layers)]
        if self.mutate_decode is not None:
            for l in range(wl.n_layers):
                self.mutate_decode(l, *ins[l])
        dins = [tuple(t.to(self.dev) for t in x) for x in ins]
        out = torch.empty((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device=self.dev)
        for t in range(S):
            for l in range(wl.n_layers):
                q, kn, vn = dins[l]
                nt0 = A.arkv_cache_progress(self.cache, l)[0]
                A.arkv_decode_step(self.cache, l, q[t], kn[t], vn[t], self.scales[l], out)
                fired = A.arkv_cache_progress(self.cache, l)[0] > nt0
                outf = A.arkv_debug_last_out_f32(self.cache, l, (wl.batch, wl.n_q_heads, wl.head_dim))
                assert np.array_equal(out.cpu().view(torch.int16).numpy().view(np.uint16), bf16_round(outf))
                over = self._gpu_scores(l) if fired else None
                for b in range(wl.batch):
                    oc = self.oracles[(l, b)]
                    qn, knn, vnn = (synth.to_numpy_f32(x[t, b]) for x in ins[l])
                    if fired:
                        # scores the oracle itself would rank on, before it adopts the GPU's
                        probe = _clone_for_scores(oc, qn, knn, vnn, self.scales[l])
                        self._check_scores(probe, l, b, over)
                    mine = None if over is None else over[b * wl.n_kv_heads:(b + 1) * wl.n_kv_heads]
                    before = copy.deepcopy(oc) if (fired and not self.lockstep) else None
                    ref, ofired = oc.decode_step(qn, knn, vnn, self.scales[l], S_override=mine if self.lockstep else None)
                    assert ofired == fired
                    if before is not None and not self._same_choice_or_in_band(oc, l, b):
                        oc = before                   # allowed divergence: go on from the GPU's choice
                        ref, _ = oc.decode_step(qn, knn, vnn, self.scales[l], S_override=mine)
                        self.oracles[(l, b)] = oc
                    for h in range(wl.n_q_heads):
                        self.max_err["out"] = max(self.max_err["out"], rel_err(outf[b, h], ref[h]))
                if fired or t % check_every == 0 or t == S - 1:
                    self.compare_state(l)

    # ---- state comparison ------------------------------------------------------------------------
    def compare_state(self, layer):
        wl = self.wl
        ex = A.arkv_cache_export(self.cache, layer, self.cfg)
        no, nq, ne, lb = A.arkv_cache_counters(self.cache, layer, self.U)
        for b in range(wl.batch):
            oc = self.oracles[(layer, b)]
            for g in range(wl.n_kv_heads):
                u = b * wl.n_kv_heads + g
                ou = oc.units[g]
                order = np.argsort(ou.pos)
                n = len(order)
                assert ex["n_live"][u] == n, (ex["n_live"][u], n)
                assert np.array_equal(ex["pos"][u, :n], ou.pos[order])              # bit-exact: who survived
                assert np.array_equal(ex["state"][u, :n], ou.state[order].astype(np.uint8))   # and in which state
                assert (no[u], nq[u]) == oc.counts(g) and lb[u] == oc.live_bytes(g)
                assert ne[u] == oc.P + 1 - n                                       # evicted so far
                assert lb[u] <= wl.capacity * 4 * wl.head_dim                      # eq. 1, per unit
                self.max_err["s1"] = max(self.max_err["s1"], rel_err(ex["s1"][u, :n], ou.s1[order]))
                self.max_err["s2"] = max(self.max_err["s2"], rel_err(ex["s2"][u, :n], ou.s2[order]))
                st = ou.state[order]
                is_o = st == O.STATE_O
                raw = ou.raw[order]
                assert np.array_equal(ex["rows_k"][u, :n][is_o], bf16_round(raw[is_o, 0]))      # bf16 rows, bit-exact
                assert np.array_equal(ex["rows_v"][u, :n][is_o], bf16_round(raw[is_o, 1]))
                qpos = ou.pos[order][~is_o]
                if len(qpos):
                    ent = [ou.q[int(p)] for p in qpos]
                    for name, key, conv in (("codes_k", "k_codes", lambda e: O.pack_codes(e, wl.bits)),
                                            ("codes_v", "v_codes", lambda e: O.pack_codes(e, wl.bits)),
                                            ("scale_k", "k_scale", lambda e: e.view(np.uint16)),
                                            ("zero_k", "k_zero", lambda e: e.view(np.uint16)),
                                            ("scale_v", "v_scale", lambda e: e.view(np.uint16)),
                                            ("zero_v", "v_zero", lambda e: e.view(np.uint16))):
                        want = np.stack([conv(e[key]) for e in ent])
                        assert np.array_equal(ex[name][u, :n][~is_o], want), name       # codes / fp16 bits, bit-exact

    def assert_within_tol(self, stats=True):
        for k, v in self.max_err.items():
            if k == "stats" and not stats:
                continue
            assert v <= TOL, (k, v, self.max_err)


def _clone_for_scores(oc, q, kn, vn, scale):
    """Copy of an oracle cache advanced by one step WITHOUT tailoring, to read the scores the
    tailor of that step would rank on."""
    c = copy.deepcopy(oc)
    N = c.N
    c.N = 10 ** 9
    c.decode_step(q, kn, vn, scale)
    c.N = N
    return c
