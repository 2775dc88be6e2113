#!/usr/bin/env python3
"""Benchmark of the ARKV decode hot path on one MI355X.

Workload (config.workload): the third benchmark configuration, the one the metric is quoted on
(32K context): Qwen3-8B-shaped cache, 36 layers, 32 q / 8 kv heads, d=128, batch 4, prompt 32768,
budget 25 % (N = 8192), 4-bit groups of 32.  Synthetic inputs, drawn on the GPU (synth.py).

A "step" is one decode step of the whole model: one arkv_decode_step call per layer (append,
attend, score update, tailor when due), cycling through all 36 layer caches (2.8 GB of distinct
cache memory per step, so the 256 MB last-level cache cannot hold it).  The prompt is scored
(arkv_prefill_stats), the OQ ratios computed (arkv_oq_ratio) and every layer committed
(arkv_prefill_commit, first tailor) before the timed region; those phases are timed separately and
reported under "prefill".

value = layer-batch decode steps per second = n_layers * steps / seconds.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def kv_bytes_per_token(d, bits):
    c_o = 4 * d
    c_q = 2 * (d + 2) if bits == 8 else 2 * (d * bits // 8 + (d // 32) * 4)
    return c_o, c_q


def algorithmic_bytes_attend(n_o, n_q, d, G, bits):
    """Bytes the method itself must move for one unit in one decode step: every live K and V row once, each live
    token's (s1, s2) read and written (16 bytes), its position and state (4 + 1 bytes), the unit's queries and
    outputs, the appended row.  (The kernels move less than this: the score update is batched over 8 steps and
    positions / states are not read during decode; the hardware counters under profiles/ show the real traffic.)"""
    c_o, c_q = kv_bytes_per_token(d, bits)
    n_live = n_o + n_q
    return n_o * c_o + n_q * c_q + 21.0 * n_live + 2 * G * d * 2 + c_o


def stored_traffic(workload):
    """HBM bytes per launch of the attention kernel from the committed rocprofv3 counter runs
    (profiles/decode_c3_hbm_counters.txt: FETCH_SIZE and WRITE_SIZE, each scaled by the factor the same
    counter shows for a copy kernel of known size).  Not measured live: counters need rocprofv3."""
    if workload != "c3_qwen3_8b_32k_b4":
        return None
    try:
        for line in open(os.path.join(ROOT, "profiles", "decode_c3_hbm_counters.txt")):
            if line.startswith("traffic_bytes_per_launch"):
                return int(line.split("=")[1])
    except OSError:
        pass
    return None


def cpu_baseline(wl, k, v, qw, dq, scale, rho, seconds_budget=12.0):
    """The oracle as it stands on one sequence of one layer: commit + a few decode steps, timed on
    the host; scaled to layer-batch steps per second by the batch size."""
    import numpy as np
    from oracle import arkv_oracle as O
    from paper_2603_08727_amd import synth
    k0, v0, qw0 = (synth.to_numpy_f32(t) for t in (k, v, qw))
    t0 = time.perf_counter()
    a = O.window_attention(qw0, k0, scale, wl.group)
    stats = O.layer_statistics(a, wl.window)[:3]
    s1, s2 = O.prefill_accumulators(a, wl.group)
    del a
    t_score = time.perf_counter() - t0
    t0 = time.perf_counter()
    oc = O.SequenceCacheOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, W=wl.window,
                               alpha=wl.alpha, gamma=wl.gamma, bits=wl.bits)
    oc.commit(k0, v0, s1, s2, float(rho))
    t_commit = time.perf_counter() - t0
    q, kn, vn = (synth.to_numpy_f32(t) for t in dq)
    n = 0
    t0 = time.perf_counter()
    while n < q.shape[0] and (n < 4 or time.perf_counter() - t0 < seconds_budget):
        oc.decode_step(q[n], kn[n], vn[n], scale)
        n += 1
    t_dec = (time.perf_counter() - t0) / n
    try:
        import threadpoolctl
        threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        threads = os.cpu_count() or 1
    return {
        "value": 1.0 / (t_dec * wl.batch), "unit": "steps/s", "cores": int(threads), "kind": "oracle",
        "sample": f"layer 0, sequence 0 of {wl.batch}: {n} decode steps after commit "
                  f"({t_dec * 1e3:.1f} ms per sequence-step; x{wl.batch} sequences per layer-batch); "
                  f"prompt scoring {t_score:.2f} s and commit {t_commit:.2f} s for that sequence, untimed in value",
        "nproc": os.cpu_count(),
    }, stats


def quick_measure(wl, rho_force=None, steps=24, warmup=4, every_step=False, byte_budget=False, packed_weight=0,
                  wg_target=0, fill=False):
    """Prefill + commit + a short timed decode run of one workload (all its layers); returns steps/s per
    layer-batch, the attention kernel's average duration and its algorithmic bytes.  Used for the policy
    and workload variants; the headline run in main() is more thorough.  fill: first step the caches (untimed)
    up to just before their next tailor, so that the timed steps see a cache at capacity."""
    import numpy as np
    import torch
    from paper_2603_08727_amd import binding as A
    from paper_2603_08727_amd import synth
    dev = "cuda"
    L, B, Hq, Hkv, d, T, W = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.prefill, wl.window
    G, U = wl.group, wl.batch * wl.n_kv_heads
    cfg = A.arkv_config_default(n_layers=L, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                                capacity_tokens=wl.capacity, window=W, alpha=wl.alpha, gamma=wl.gamma,
                                tau=wl.tau, quant_bits=wl.bits, tailor_policy=1 if every_step else 0,
                                budget_mode=1 if byte_budget else 0)
    cache = A.arkv_cache_create(cfg)
    try:
        if packed_weight or wg_target:
            A.arkv_debug_set_launch_shape(cache, wg_target, packed_weight, 0)
        scales = [synth.softmax_scale(wl, l) for l in range(L)]
        stats = torch.zeros((L, B, 3), dtype=torch.float32, device=dev)
        for l in range(L):
            k, v, qw = synth.prefill_inputs(wl, l, device=dev)
            A.arkv_prefill_stats(cache, l, qw, k, T, scales[l], stats[l])
            del k, v, qw
        rho = A.arkv_oq_ratio(stats.cpu().numpy(), wl.tau)
        if rho_force is not None:
            rho = np.full_like(rho, rho_force)
        for l in range(L):
            k, v, qw = synth.prefill_inputs(wl, l, device=dev)
            A.arkv_prefill_commit(cache, l, k, v, T, rho[l])
            del k, v, qw
        total = warmup + 2 * steps
        n_fill = 0
        if fill:
            live = A.arkv_cache_progress(cache, 0)[1]
            n_fill = max(0, wl.capacity - 2 - live - total)          # the timed steps end one step short of the tailor
        per_layer = [synth.decode_inputs(wl, l, total, device=dev) for l in range(L)]
        q_all = torch.stack([p[0] for p in per_layer], dim=1).contiguous()
        kn_all = torch.stack([p[1] for p in per_layer], dim=1).contiguous()
        vn_all = torch.stack([p[2] for p in per_layer], dim=1).contiguous()
        del per_layer
        out = torch.empty((L, B, Hq, d), dtype=torch.bfloat16, device=dev)
        lib = A.load()
        stream = torch.cuda.current_stream().cuda_stream
        qs_, ks_, os_ = B * Hq * d * 2, B * Hkv * d * 2, B * Hq * d * 2
        qp, kp, vp, op = q_all.data_ptr(), kn_all.data_ptr(), vn_all.data_ptr(), out.data_ptr()
        t_i = 0

        def run(n):
            nonlocal t_i
            for _ in range(n):
                t = t_i % total                       # (the filling steps reuse the drawn inputs)
                for l in range(L):
                    rc = lib.arkv_decode_step(cache, l, qp + (t * L + l) * qs_, kp + (t * L + l) * ks_,
                                              vp + (t * L + l) * ks_, float(scales[l]), op + l * os_, stream)
                    if rc != 0:
                        raise A.ArkvError(rc, "arkv_decode_step")
                t_i += 1

        run(n_fill)
        run(warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        no = nq = 0.0
        for l in range(L):
            a_, b_, _, _ = A.arkv_cache_counters(cache, l, U)
            no += a_.sum(); nq += b_.sum()
        no /= L * U; nq /= L * U
        A.arkv_debug_time_attend(cache, True)
        run(steps)
        ms, n = A.arkv_debug_attend_time(cache)
        A.arkv_debug_time_attend(cache, False)
        bpl = U * algorithmic_bytes_attend(no + steps / 2.0, nq, d, G, wl.bits)
        us = ms * 1e3 / max(n, 1)
        return {"steps_per_s_per_layer_batch": round(L * steps / dt, 1), "attend_us": round(us, 2),
                "algorithmic_MB_per_launch": round(bpl / 1e6, 2), "achieved_GBps": round(bpl / (us * 1e-6) / 1e9, 1),
                "frac_of_hbm_peak": round(bpl / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                "tokens_per_unit": {"original": round(float(no), 1), "quantized": round(float(nq), 1)},
                "capacity_tokens": wl.capacity, "context": T, "n_layers": L, "batch": B, "quant_bits": wl.bits,
                "us_per_call": round(dt / (L * steps) * 1e6, 2), "tailor_every_step": bool(every_step),
                "tailors_so_far_layer0": A.arkv_cache_progress(cache, 0)[0]}
    finally:
        A.arkv_cache_destroy(cache)


def scorer_measure(wl, window, layers=4):
    """Prefill scorer alone (window logits, causal softmax, column sums, the three statistics) on `layers`
    layers of a workload with the observation window set to `window`: time per layer against both roofs."""
    import torch
    from paper_2603_08727_amd import binding as A
    from paper_2603_08727_amd import synth
    wl = wl.scaled(n_layers=layers, window=window)
    dev = "cuda"
    L, B, Hq, Hkv, d, T, W = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.prefill, wl.window
    cfg = A.arkv_config_default(n_layers=L, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                                capacity_tokens=wl.capacity, window=W, alpha=wl.alpha, gamma=wl.gamma,
                                tau=wl.tau, quant_bits=wl.bits)
    cache = A.arkv_cache_create(cfg)
    try:
        stats = torch.zeros((L, B, 3), dtype=torch.float32, device=dev)
        ms = []
        for rep in range(2):                  # second round: warm code, same work
            if rep:
                A.arkv_cache_reset(cache, -1)
            for l in range(L):
                k, v, qw = synth.prefill_inputs(wl, l, device=dev)
                del v
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                A.arkv_prefill_stats(cache, l, qw, k, T, synth.softmax_scale(wl, l), stats[l])
                e1.record()
                torch.cuda.synchronize()
                if rep:
                    ms.append(e0.elapsed_time(e1))
                del k, qw
        t = sum(ms) / len(ms) * 1e-3
        flops = 2.0 * W * Hq * T * d * B      # one pass of the window logits; the kernels make two
        kbytes = B * Hkv * T * d * 2
        t_hbm, t_mfma = kbytes / (HBM_PEAK_GBPS * 1e9), flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        return {"window": W, "query_rows_per_unit": W * (Hq // Hkv), "ms_per_layer": round(t * 1e3, 4),
                "TFLOPs_one_pass": round(flops / t / 1e12, 1), "TFLOPs_executed_two_passes": round(2 * flops / t / 1e12, 1),
                "frac_of_bf16_mfma_peak_executed": round(2 * flops / t / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "GBps_keys_once": round(kbytes / t / 1e9, 1),
                "roof_us_keys_once_at_hbm_peak": round(t_hbm * 1e6, 1), "roof_us_one_pass_at_mfma_peak": round(t_mfma * 1e6, 1),
                "bound": "hbm" if t_hbm > t_mfma else "mfma",
                "frac_of_min_roof": round(max(t_hbm, t_mfma) / t, 4),
                "batch": B, "context": T, "layers_timed": L}
    finally:
        A.arkv_cache_destroy(cache)


def attention_measure(wl, layers=2):
    """Causal prefill attention of the whole prompt (one call per layer) with the scorer fused, against the
    bf16 matrix-core peak, and the scorer's cost with and without the fusion."""
    import torch
    from paper_2603_08727_amd import binding as A
    from paper_2603_08727_amd import synth
    wl = wl.scaled(n_layers=layers)
    dev = "cuda"
    L, B, Hq, Hkv, d, T, W = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.prefill, wl.window
    cfg = A.arkv_config_default(n_layers=L, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                                capacity_tokens=wl.capacity, window=W, alpha=wl.alpha, gamma=wl.gamma,
                                tau=wl.tau, quant_bits=wl.bits)
    cache = A.arkv_cache_create(cfg)
    try:
        res = {}
        for name, with_stats in (("attention_only", False), ("attention_with_scorer", True)):
            ms = []
            for rep in range(2):
                A.arkv_cache_reset(cache, -1)
                for l in range(L):
                    k, v, qw = synth.prefill_inputs(wl, l, device=dev)
                    g = torch.Generator(device=dev).manual_seed(wl.seed + 1000 * l + 77)
                    q = torch.randn((B, Hq, T, d), generator=g, device=dev).to(torch.bfloat16)
                    q[:, :, T - W:, :] = qw
                    out = torch.empty_like(q)
                    stats = torch.zeros((B, 3), dtype=torch.float32, device=dev) if with_stats else None
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    A.arkv_prefill_attention(cache, l, q, k, v, T, T, synth.softmax_scale(wl, l), out, stats)
                    e1.record()
                    torch.cuda.synchronize()
                    if rep:
                        ms.append(e0.elapsed_time(e1))
                    del q, k, v, out
            res[name] = sum(ms) / len(ms)
        flops = 4.0 * B * Hq * d * (T * (T + 1) / 2.0)          # QK^T and PV over the causal half
        t = res["attention_only"] * 1e-3
        return {"ms_per_layer_attention": round(res["attention_only"], 3),
                "ms_per_layer_attention_with_scorer": round(res["attention_with_scorer"], 3),
                "scorer_extra_ms_when_fused": round(res["attention_with_scorer"] - res["attention_only"], 3),
                "TFLOPs": round(flops / t / 1e12, 1), "frac_of_bf16_mfma_peak": round(flops / t / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "context": T, "batch": B, "layers_timed": L}
    finally:
        A.arkv_cache_destroy(cache)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="c3_qwen3_8b_32k_b4")
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers (debug)")
    ap.add_argument("--prefill", type=int, default=None, help="override the prompt length (debug)")
    ap.add_argument("--budget", type=float, default=None, help="override the budget fraction (debug)")
    ap.add_argument("--rho", type=float, default=None, help="force every layer's OQ ratio (variant runs)")
    ap.add_argument("--alpha", type=float, default=None, help="override the slack factor (debug, ceiling runs)")
    ap.add_argument("--bits", type=int, default=None, help="override the Quantized format: 2, 4 or 8 (variant runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=8)
    ap.add_argument("--no-tailor-run", action="store_true", help="skip stepping 4 layers up to their next tailor")
    ap.add_argument("--no-variants", action="store_true", help="skip the policy / other-workload variant runs")
    ap.add_argument("--scorer-only", type=int, default=0, metavar="W",
                    help="time only the prefill scorer of the scorer-stress configuration with an observation window of W "
                         "tokens and print that entry (profiling runs)")
    ap.add_argument("--attention-only", action="store_true",
                    help="time only the causal prefill attention of the workload's prompt and print that entry")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU (units of the cache never interact across GPUs; "
              "sharding by kv-head or sequence is a design note, not built); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2603_08727_amd import binding as A
    from paper_2603_08727_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda"
    wl = synth.CONFIGS[args.workload]
    if args.layers:
        wl = wl.scaled(n_layers=args.layers)
    if args.prefill:
        wl = wl.scaled(prefill=args.prefill)
    if args.budget:
        wl = wl.scaled(budget_frac=args.budget)
    if args.alpha:
        wl = wl.scaled(alpha=args.alpha)
    if args.bits:
        wl = wl.scaled(bits=args.bits)
    if args.scorer_only:
        print(json.dumps({"scorer_stress": scorer_measure(synth.C5, args.scorer_only), "workload": synth.C5.name}))
        return
    if args.attention_only:
        print(json.dumps({"prefill_attention": attention_measure(wl), "workload": wl.name}))
        return
    L, B, Hq, Hkv, d, T, W = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.prefill, wl.window
    G, U = wl.group, wl.batch * wl.n_kv_heads
    total_steps = args.warmup + args.steps + args.profile_steps + 8
    cfg = A.arkv_config_default(n_layers=L, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                                capacity_tokens=wl.capacity, window=W, alpha=wl.alpha, gamma=wl.gamma,
                                tau=wl.tau, quant_bits=wl.bits)
    cache = A.arkv_cache_create(cfg)
    scales = [synth.softmax_scale(wl, l) for l in range(L)]

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- prefill scorer when the caller's attention kernel supplies the window rows' log-sum-exp (a few layers;
    # the normalisers come from torch here and are not timed) ---------------------------------------------
    def window_lse(qw, k, scale):
        out = torch.empty((B, Hq, W), dtype=torch.float32, device=dev)
        vis = torch.arange(T, device=dev)[None, :] <= (T - W + torch.arange(W, device=dev))[:, None]      # [W][T]
        for b in range(B):
            for g in range(Hkv):
                lg = (qw[b, g * G:(g + 1) * G].float().reshape(G * W, d) @ k[b, g].float().T) * scale
                lg = lg.reshape(G, W, T).masked_fill(~vis[None], float("-inf"))
                out[b, g * G:(g + 1) * G] = torch.logsumexp(lg, dim=-1)
        return out

    t_lse_l = []
    stats_lse = torch.zeros((B, 3), dtype=torch.float32, device=dev)
    for l in range(min(L, 4)):
        k, v, qw = synth.prefill_inputs(wl, l, device=dev)
        lse = window_lse(qw, k, scales[l])
        for _ in range(2):
            e0, e1 = ev(), ev()
            e0.record()
            A.arkv_prefill_stats_lse(cache, l, qw, k, T, scales[l], lse, stats_lse)
            e1.record()
            torch.cuda.synchronize()
        t_lse_l.append(e0.elapsed_time(e1))
        del k, v, qw, lse
    # ---- prefill scorer, all layers -------------------------------------------------------------
    stats = torch.zeros((L, B, 3), dtype=torch.float32, device=dev)
    t_stats_l = []
    sample = None
    for l in range(L):
        k, v, qw = synth.prefill_inputs(wl, l, device=dev)
        if l == 0:
            sample = (k[0].cpu(), v[0].cpu(), qw[0].cpu())
        e0, e1 = ev(), ev()
        e0.record()
        A.arkv_prefill_stats(cache, l, qw, k, T, scales[l], stats[l])
        e1.record()
        torch.cuda.synchronize()
        t_stats_l.append(e0.elapsed_time(e1))
        del k, v, qw
    # per-layer figure = the median over the layers: the first calls of a process pay one-off costs (code
    # objects, clocks), reported separately
    t_stats = float(np.median(t_stats_l)) * L
    stats_h = stats.cpu().numpy()
    rho = A.arkv_oq_ratio(stats_h, wl.tau)
    if args.rho is not None:
        rho = np.full_like(rho, args.rho)
    # ---- commit ---------------------------------------------------------------------------------
    t_commit_l = []
    for l in range(L):
        k, v, qw = synth.prefill_inputs(wl, l, device=dev)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        A.arkv_prefill_commit(cache, l, k, v, T, rho[l])
        torch.cuda.synchronize()
        t_commit_l.append((time.perf_counter() - t0) * 1e3)
        del k, v, qw
    t_commit = float(np.median(t_commit_l)) * L
    # ---- decode inputs [S][L][B][H][d] ------------------------------------------------------------
    per_layer = [synth.decode_inputs(wl, l, total_steps, device=dev) for l in range(L)]
    q_all = torch.stack([p[0] for p in per_layer], dim=1).contiguous()
    kn_all = torch.stack([p[1] for p in per_layer], dim=1).contiguous()
    vn_all = torch.stack([p[2] for p in per_layer], dim=1).contiguous()
    dq_sample = tuple(p[:, 0].cpu() for p in per_layer[0])
    del per_layer
    out = torch.empty((L, B, Hq, d), dtype=torch.bfloat16, device=dev)
    step_i = 0

    # raw pointers once: the timed loop is one C call per layer with no tensor bookkeeping in between
    lib = A.load()
    stream = torch.cuda.current_stream().cuda_stream
    qs_, ks_, os_ = B * Hq * d * 2, B * Hkv * d * 2, B * Hq * d * 2
    qp, kp, vp, op = q_all.data_ptr(), kn_all.data_ptr(), vn_all.data_ptr(), out.data_ptr()
    sc_f = [float(x) for x in scales]

    def one_step():
        nonlocal step_i
        t = step_i
        for l in range(L):
            rc = lib.arkv_decode_step(cache, l, qp + (t * L + l) * qs_, kp + (t * L + l) * ks_,
                                      vp + (t * L + l) * ks_, sc_f[l], op + l * os_, stream)
            if rc != 0:
                raise A.ArkvError(rc, "arkv_decode_step")
        step_i += 1

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    no0 = np.zeros(L); nq0 = np.zeros(L); ne0 = np.zeros(L)
    for l in range(L):
        a_, b_, e_, _ = A.arkv_cache_counters(cache, l, U)
        no0[l], nq0[l], ne0[l] = a_.sum(), b_.sum(), e_.sum()
    # composition of the caches after the first tailor (the quantities of Table VII, here for the synthetic
    # statistics of this workload): Quantized tokens over the capacity, evicted tokens over all tokens seen
    composition = {"quant_ratio_of_capacity": round(float(nq0.sum() / (L * U * wl.capacity)), 4),
                   "evict_ratio_of_tokens_seen": round(float(ne0.sum() / max(no0.sum() + nq0.sum() + ne0.sum(), 1.0)), 4),
                   "layers_all_original": int((nq0 == 0).sum()), "n_layers": L}
    tailors0 = sum(A.arkv_cache_progress(cache, l)[0] for l in range(L))
    # ---- timed region -----------------------------------------------------------------------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    tailors1 = sum(A.arkv_cache_progress(cache, l)[0] for l in range(L))
    ms_per_step = elapsed * 1e3 / args.steps
    value = L * args.steps / elapsed

    # ---- dominant kernel: live duration by HIP events on the launch stream -------------------------
    A.arkv_debug_time_attend(cache, True)
    no_p = np.zeros(L); nq_p = np.zeros(L)
    for l in range(L):
        a_, b_, _, _ = A.arkv_cache_counters(cache, l, U)
        no_p[l], nq_p[l] = a_.sum(), b_.sum()
    for _ in range(args.profile_steps):
        one_step()
    att_ms, att_n = A.arkv_debug_attend_time(cache)
    A.arkv_debug_time_attend(cache, False)
    # tokens per launch during the profiled steps: counts before + half the appended tokens
    mean_no = (no_p.mean() + U * args.profile_steps / 2.0) / U
    mean_nq = nq_p.mean() / U
    bytes_per_launch = U * algorithmic_bytes_attend(mean_no, mean_nq, d, G, wl.bits)
    att_us = att_ms * 1e3 / max(att_n, 1)
    achieved = bytes_per_launch / (att_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "kernel": "k_decode_attend", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": stored_traffic(wl.name),
                "avg_kernel_us": round(att_us, 2), "launches_timed": int(att_n),
                "avg_kernel_us_clock": "HIP event pair around every launch of the kernel on the launch stream "
                                       "(arkv_debug_time_attend); agrees with rocprofv3's kernel trace.  It may exceed "
                                       "step.us_per_layer_batch_call (stream time per call without events): an event "
                                       "pair costs ~2 us that back-to-back launches do not pay, and consecutive "
                                       "launches overlap their start-up with the previous launch's tail",
                "algorithmic_bytes_per_launch": int(bytes_per_launch),
                "tokens_per_unit": {"original": round(float(mean_no), 1), "quantized": round(float(mean_nq), 1)}}
    # whole-step view: algorithmic bytes of a layer-batch call over its wall time in the timed region
    mean_no_t = (no0.mean() + U * args.steps / 2.0) / U
    mean_nq_t = nq0.mean() / U
    step_bytes = U * algorithmic_bytes_attend(mean_no_t, mean_nq_t, d, G, wl.bits)
    call_us = elapsed * 1e6 / (L * args.steps)

    # ---- variant: all layers in one launch ----------------------------------------------------------
    variants = {}
    if L <= 64:
        sc = np.array(scales, dtype=np.float32)
        for _ in range(2):
            A.arkv_decode_step_layers(cache, 0, L, q_all[step_i], kn_all[step_i], vn_all[step_i], sc, out); step_i += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        nv = 4
        for _ in range(nv):
            A.arkv_decode_step_layers(cache, 0, L, q_all[step_i], kn_all[step_i], vn_all[step_i], sc, out); step_i += 1
        torch.cuda.synchronize()
        tv = time.perf_counter() - t0
        variants["all_layers_one_launch"] = {"steps_per_s_per_layer_batch": round(L * nv / tv, 1),
                                             "achieved_GBps": round(L * step_bytes * nv / tv / 1e9, 1)}

    # ---- practical ceiling: plain streaming read of the same number of bytes per launch ---------------
    ceiling = None
    try:
        big = torch.empty(3 << 30, dtype=torch.uint8, device=dev)
        bpl = max(524288, int(bytes_per_launch) // 524288 * 524288)
        us = A.arkv_measure_stream_read(big, bpl, 200, 0)
        us1 = A.arkv_measure_stream_read(big, bpl, 200, 1)
        A.arkv_measure_stream_read(big, bpl, 20, 2)      # known-size copy: calibrates the write counter under rocprofv3
        ceiling = {"us_per_launch": round(us, 2), "GBps": round(bpl / (us * 1e-6) / 1e9, 1), "bytes_per_launch": bpl,
                   "operand_layout_GBps": round(bpl / (us1 * 1e-6) / 1e9, 1)}
        roofline["frac_of_stream_read_ceiling"] = round(achieved / ceiling["GBps"], 4)
        del big
    except Exception as e:  # noqa: BLE001 - the ceiling is informative only
        ceiling = {"error": str(e)}

    # ---- tailor at its natural cadence: step a few layers until the cache is full -----------------------
    tailor = None
    if not args.no_tailor_run:
        nl = min(L, 4)
        N = wl.capacity
        live = A.arkv_cache_progress(cache, 0)[1]
        # all layers are in the same state; bring the first nl to the step that fills the cache
        plain_ms, tailor_ms, n_plain = 0.0, 0.0, 0
        t_idx = step_i
        while live < N - 1:
            t = t_idx % total_steps
            for l in range(nl):
                lib.arkv_decode_step(cache, l, qp + (t * L + l) * qs_, kp + (t * L + l) * ks_,
                                     vp + (t * L + l) * ks_, sc_f[l], op + l * os_, stream)
            live += 1; t_idx += 1
        torch.cuda.synchronize()
        t = t_idx % total_steps
        for l in range(nl):
            e0, e1 = ev(), ev()
            e0.record()
            lib.arkv_decode_step(cache, l, qp + (t * L + l) * qs_, kp + (t * L + l) * ks_,
                                 vp + (t * L + l) * ks_, sc_f[l], op + l * os_, stream)
            e1.record()
            torch.cuda.synchronize()
            tailor_ms += e0.elapsed_time(e1)
        fired = all(A.arkv_cache_progress(cache, l)[0] == 2 for l in range(nl))
        # the same layers right after their tailor (cache back at W + b tokens, counts re-read from the device)
        def run_after(nsteps):
            nonlocal t_idx
            for _ in range(nsteps):
                t_idx += 1
                t_ = t_idx % total_steps
                for l in range(nl):
                    lib.arkv_decode_step(cache, l, qp + (t_ * L + l) * qs_, kp + (t_ * L + l) * ks_,
                                         vp + (t_ * L + l) * ks_, sc_f[l], op + l * os_, stream)
        run_after(8)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_after(32)
        torch.cuda.synchronize()
        after_us = (time.perf_counter() - t0) / (32 * nl) * 1e6
        cadence = N - (min(int(np.floor(np.float32(wl.alpha) * (N - W))), N - W - 1) + W)
        tailor = {"layers_stepped": nl, "fired": bool(fired), "step_with_tailor_us": round(tailor_ms * 1e3 / nl, 1),
                  "cadence_steps": int(cadence), "us_per_call_after_tailor": round(after_us, 2),
                  "amortised_us_per_step": round((tailor_ms * 1e3 / nl - call_us) / max(cadence, 1), 3)}

    result = {
        "metric": "decode steps/sec per layer-batch at 32K ctx; achieved HBM GB/s vs peak", "value": round(value, 1), "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "n_layers": L, "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": d, "context": T, "capacity_tokens": wl.capacity, "quant_bits": wl.bits,
                   "window": W, "launch": "one arkv_decode_step per layer",
                   "rows": "bf16 Original, %s Quantized; logits on bf16 MFMA, softmax and PV in f32" % ("fp8" if wl.bits == 8 else "int%d" % wl.bits)},
        "roofline": roofline,
        "step": {"us_per_layer_batch_call": round(call_us, 2),
                 "achieved_GBps_whole_call": round(step_bytes / (call_us * 1e-6) / 1e9, 1),
                 "frac_of_hbm_peak_whole_call": round(step_bytes / (call_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                 "tailors_in_timed_region": int(tailors1 - tailors0)},
        "cache_composition": composition,
        "prefill": {"scorer_ms_per_layer": round(t_stats / L, 3), "scorer_ms_first_layer": round(t_stats_l[0], 3),
                    "scorer_ms_per_layer_log_sum_exp_supplied": round(float(np.median(t_lse_l)), 3),
                    "scorer_TFLOPs": round(2.0 * W * Hq * T * d * B / (t_stats / L * 1e-3) / 1e12, 1),
                    "scorer_frac_of_bf16_mfma_peak": round(2.0 * W * Hq * T * d * B / (t_stats / L * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                    "scorer_GBps_keys_once": round((B * Hkv * T * d * 2) / (t_stats / L * 1e-3) / 1e9, 1),
                    # the keys are streamed twice by necessity (a probability needs its row's maximum and sum first)
                    "scorer_frac_of_hbm_peak_two_passes": round(2 * (B * Hkv * T * d * 2) / (t_stats / L * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                    "commit_ms_per_layer": round(t_commit / L, 3), "commit_ms_first_layer": round(t_commit_l[0], 3),
                    "rho_min_mean_max": [round(float(rho.min()), 3), round(float(rho.mean()), 3), round(float(rho.max()), 3)]},
        "variants": variants,
        "stream_read_ceiling": ceiling,
        "tailor": tailor,
    }
    A.arkv_cache_destroy(cache)
    cache = None
    del q_all, kn_all, vn_all
    torch.cuda.empty_cache()
    if not args.no_variants:
        # kernel-level counterpart of the paper's baselines (Sec. V-C) on the same 32K-context shape, 12 layers:
        # full cache (no limit), evict-only (rho = 1), quantise-all-kept (rho = 0), and a mixed cache (rho = 0.5)
        base12 = wl.scaled(n_layers=min(L, 12))
        full = base12.scaled(budget_frac=(T + 128) / T)
        pol = {
            "base_full_cache": quick_measure(full),
            "origin_evict_only_rho1": quick_measure(base12, rho_force=1.0),
            "quant_all_kept_rho0": quick_measure(base12, rho_force=0.0),
            "arkv_mixed_rho0.5": quick_measure(base12, rho_force=0.5),
            "arkv_scored_rho": quick_measure(base12),
            "quant_all_kept_rho0_fp8_rows": quick_measure(base12.scaled(bits=8), rho_force=0.0),
            "arkv_mixed_rho0.5_fp8_rows": quick_measure(base12.scaled(bits=8), rho_force=0.5),
            "arkv_mixed_rho0.5_byte_budget": quick_measure(base12, rho_force=0.5, byte_budget=True),
            "arkv_scored_rho_tailor_every_step": quick_measure(base12.scaled(n_layers=4), every_step=True),
            # the paper's composition (Table VII: Quantized tokens = 14.4 % of the budget): n_q = 0.144 N = 1180 of
            # the b = 6120 survivors, i.e. rho = (6120 - 1180) / 8160
            "arkv_paper_like_composition_rho0.605": quick_measure(base12, rho_force=0.6054),
            # cache at capacity (just before a tailor) at rho = 0.5: 8190 tokens per unit, 2040 of them Quantized
            "arkv_mixed_rho0.5_at_capacity": quick_measure(base12, rho_force=0.5, fill=True),
            # ceiling runs of the packed-row stream: almost the whole 32K prompt kept, all of it Quantized
            "ceiling_all_quantized_32k": quick_measure(base12.scaled(n_layers=6, budget_frac=0.99, alpha=0.99), rho_force=0.0),
            "ceiling_all_quantized_32k_fp8_rows": quick_measure(base12.scaled(n_layers=6, budget_frac=0.99, alpha=0.99, bits=8), rho_force=0.0),
            "ceiling_all_quantized_32k_2bit_rows": quick_measure(base12.scaled(n_layers=6, budget_frac=0.99, alpha=0.99, bits=2), rho_force=0.0),
        }
        ref = pol["base_full_cache"]["steps_per_s_per_layer_batch"]
        for v_ in pol.values():
            v_["relative_to_full_cache"] = round(v_["steps_per_s_per_layer_batch"] / ref, 3)
        result["policies"] = pol
        # the other decode configurations (8 layers each), same measurement
        result["other_workloads"] = {
            "c2_llama3_8b_8k": quick_measure(synth.C2.scaled(n_layers=8)),
            "c4_llama3_8b_128k_2bit": quick_measure(synth.C4),          # all 32 layers (the first 8 hold no Quantized rows)
            "c4_llama3_8b_128k_2bit_rho0.5": quick_measure(synth.C4.scaled(n_layers=8), rho_force=0.5),
            "c4_shape_all_original_100pct": quick_measure(synth.C4.scaled(n_layers=4, budget_frac=(synth.C4.prefill + 128) / synth.C4.prefill)),
        }
    if not args.no_variants:
        # prefill-scorer stress shape (16K context, batch 8) at the paper's window and at a 4x window, where the
        # contraction is compute-bound
        result["scorer_stress"] = {"c5_w32": scorer_measure(synth.C5, 32), "c5_w128": scorer_measure(synth.C5, 128)}
        # causal prefill attention of the 32K prompt with the scorer fused (the headline workload's prompt)
        result["prefill_attention"] = attention_measure(wl)
    if not args.no_cpu_baseline:
        # the oracle needs ~10 ms per sequence-step at this shape: 1500 steps of sequence 0 bound the sample
        # to the time budget below (same recipe as the GPU run's decode inputs, a longer draw)
        dq_sample = tuple(p[:, 0].cpu() for p in synth.decode_inputs(wl, 0, 1500, device=dev))
        cb, ref_stats = cpu_baseline(wl, *sample, dq_sample, scales[0], rho[0, 0])
        result["cpu_baseline"] = cb
        got = stats_h[0, 0]
        result["prefill"]["stats_rel_err_vs_oracle_layer0_seq0"] = [
            float(abs(got[i] - ref_stats[i]) / max(abs(ref_stats[i]), 1e-300)) for i in range(3)]
    print(json.dumps(result))


if __name__ == "__main__":
    main()
