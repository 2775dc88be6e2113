"""Where the time of one decode launch goes: in-kernel timestamps of a profiling build.

Usage (GPU; build first with `python -m paper_2603_08727_amd.build --phase-trace`):
    python -m paper_2603_08727_amd.phase_trace [--workload c3|c4] [--layers N] [--rho R] [--steps K]

Runs the prompt phase and K decode steps of N layers of the workload on the profiling library, then reads the
100 MHz timestamps that thread 0 of every workgroup of the LAST decode launch stored at its phase boundaries
(arkv_debug_phase_trace) and prints, per phase, the distribution over the workgroups, per XCD the tile loop's
duration, and the merge's own phases in the merging workgroups.  The last launch is a read-only one when K % 8 != 0
and one that also updates the scores when K % 8 == 0 (the update runs on every 8th step after the commit).
"""
from __future__ import annotations

import argparse
import os
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
os.environ["ARKV_LIBRARY"] = os.path.join(_HERE, "libarkv_trace.so")   # before the binding is imported

import numpy as np   # noqa: E402
import torch         # noqa: E402

sys.path.insert(0, os.path.dirname(_HERE))
from paper_2603_08727_amd import binding as A, synth   # noqa: E402

PHASES = ["start", "first tile requested", "bf16 rows", "new token", "packed rows", "reduce + partial stored",
          "ticket (+ merge)"]
MERGE_PHASES = ["partial stored -> merge entered (acknowledgements, ticket)", "loads issued", "weights reduced",
                "barrier", "accumulated", "stored"]


def dist(x):
    return "min %6.2f  med %6.2f  p90 %6.2f  max %6.2f" % (x.min(), np.median(x), np.percentile(x, 90), x.max())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c3", choices=["c3", "c4"])
    ap.add_argument("--layers", type=int, default=6)
    ap.add_argument("--rho", type=float, default=None, help="force this OQ ratio in every layer")
    ap.add_argument("--steps", type=int, default=12)
    args = ap.parse_args()
    if not os.path.exists(os.environ["ARKV_LIBRARY"]):
        sys.exit("libarkv_trace.so is missing: python -m paper_2603_08727_amd.build --phase-trace")
    wl = (synth.C4 if args.workload == "c4" else synth.C3).scaled(n_layers=args.layers)
    L, B, Hq, Hkv, d, T, W = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.prefill, wl.window
    cfg = A.arkv_config_default(n_layers=L, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                                capacity_tokens=wl.capacity, window=W, alpha=wl.alpha, gamma=wl.gamma, tau=wl.tau,
                                quant_bits=wl.bits)
    cache = A.arkv_cache_create(cfg)
    scales = [synth.softmax_scale(wl, l) for l in range(L)]
    stats = torch.zeros((L, B, 3), dtype=torch.float32, device="cuda")
    for l in range(L):
        k, v, qw = synth.prefill_inputs(wl, l, device="cuda")
        A.arkv_prefill_stats(cache, l, qw, k, T, scales[l], stats[l])
    rho = A.arkv_oq_ratio(stats.cpu().numpy(), wl.tau)
    if args.rho is not None:
        rho = np.full_like(rho, args.rho)
    for l in range(L):
        k, v, qw = synth.prefill_inputs(wl, l, device="cuda")
        A.arkv_prefill_commit(cache, l, k, v, T, rho[l])
    out = torch.empty((B, Hq, d), dtype=torch.bfloat16, device="cuda")
    dq = [synth.decode_inputs(wl, l, args.steps, device="cuda") for l in range(L)]
    for t in range(args.steps):
        for l in reversed(range(L)):      # layer 0 last: its launch is the one the trace keeps
            A.arkv_decode_step(cache, l, dq[l][0][t], dq[l][1][t], dq[l][2][t], scales[l], out)
    torch.cuda.synchronize()

    U = B * Hkv
    big = A.arkv_debug_phase_trace(0, 8192)
    mk = big[8190].astype(np.int64)
    # rows the last launch wrote are the ones stamped between its two marker kernels (row = unit * splits + split)
    inside = (big[:8190, 0].astype(np.int64) >= mk[0]) & (big[:8190, 6].astype(np.int64) <= mk[1])
    n = int(np.count_nonzero(inside))
    assert n > 0 and inside[:n].all() and n % U == 0, "unexpected trace contents"
    t = big[:n, :7].astype(np.int64)
    rel = (t - t[:, 0].min()) * 0.01    # microseconds
    print("workload %s, %d layers, rho %s, last launch of step %d (%s): %d workgroups = %d units x %d splits" % (
        wl.name, L, "scored" if args.rho is None else args.rho, args.steps,
        "with score update" if args.steps % 8 == 0 else "read-only", n, U, n // U))
    print("marker kernel before -> first workgroup starts %.2f us; last workgroup ends -> marker kernel after %.2f us; "
          "marker to marker %.2f us" % ((t[:, 0].min() - mk[0]) * 0.01, (mk[1] - t[:, 6].max()) * 0.01,
                                       (mk[1] - mk[0]) * 0.01))
    print("last workgroup ends %.2f us after the first started" % rel[:, 6].max())
    print("%-28s %s" % ("workgroup start", dist(rel[:, 0])))
    for i in range(1, 7):
        print("%-28s %s   | ends at med %6.2f max %6.2f" % (PHASES[i], dist(rel[:, i] - rel[:, i - 1]),
                                                            np.median(rel[:, i]), rel[:, i].max()))
    xcc = big[:n, 7].astype(np.int64) & 0xF
    loop = rel[:, 4] - rel[:, 1]
    for x in sorted(set(xcc.tolist())):
        m = xcc == x
        print("  XCD %d: %3d workgroups | first tile requested after med %.2f | tile loops med %.2f p90 %.2f | "
              "loops end med %.2f max %.2f" % (x, m.sum(), np.median((rel[:, 1] - rel[:, 0])[m]), np.median(loop[m]),
                                               np.percentile(loop[m], 90), np.median(rel[m, 4]), rel[m, 4].max()))
    mt = A.arkv_debug_phase_trace(1, 8192)[:n].astype(np.int64)
    merging = mt[:, 0] > t[:, 5]
    print("merging workgroups: %d" % merging.sum())
    prev = t[merging, 5]
    for i, name in enumerate(MERGE_PHASES):
        dcol = (mt[merging, i] - prev) * 0.01
        print("  %-58s med %.2f max %.2f" % (name, np.median(dcol), dcol.max()))
        prev = mt[merging, i]
    A.arkv_cache_destroy(cache)


if __name__ == "__main__":
    main()
