"""CPU oracle for the ARKV hot path (test infrastructure, NOT a product path).

A plain, slow, obviously-correct NumPy implementation of what the paper's
per-layer KV-cache manager computes.  Only tests/, __graft_entry__.smoke()
and the cpu_baseline leg of bench.py may import it; the HIP library never
does, and this file imports nothing from the HIP package.  It shares no code,
table or helper with the GPU path.

Arithmetic is fp64 unless a function says otherwise.  Two places are fp32 by
design, because an integer decision hangs on them and both sides must take it
in the same precision:
  * quantize_groups and quantize_fp8_rows (codes / fp16 scale / fp16 zero),
  * hh_score(..., exact32=True)  (selection keys).

What follows the paper, by passage:
  window_attention        Sec. IV-C, eq. 2   (observation window, causal softmax)
  causal_attention_rows   the causal prefill attention eq. 2 is a slice of (Sec. IV-C, first paragraph)
  window_lse              the normalisers of eq. 2's rows (log of the softmax denominators)
  layer_statistics        Sec. IV-C, eqs. 3-5 (entropy, variance, kurtosis)
  prefill_accumulators    Sec. IV-E, eq. 9   (first samples of the per-token moments)
  oq_score / oq_ratio     Sec. IV-D, eqs. 6-7
  budget_counts           Sec. IV-D eq. 8, Alg. 1 "Assign origin budget", Sec. IV-F eq. 10 (b)
  hh_score                Sec. IV-E, eq. 9
  tailor_assign           Sec. IV-F, eq. 10; Alg. 1 "Decoding Phase"
  quantize_* / dequantize Alg. 1 "Reconstruction Before Attention" (uniform
                          low-bit scheme of the benchmark configs, groups of 32)
  quantize_fp8_rows / dequantize_fp8_row
                          the same passage in the paper's own format: fp8 codes
                          with one scale per token row, x~ = q^ * s
  SequenceCacheOracle     Alg. 1 end to end for one (layer, sequence)

Readings taken where the paper is silent or garbled (numbered R1, R2, ...) are
repeated at the function they affect.

Parity pins (tests/test_oracle_*.py): brute-force loops on tiny inputs, closed
forms for the statistics, library routines for special cases (softmax
attention, entropy, kurtosis), invariants of the selection and of the budget,
half-step bound of the quantiser.  Unpinned: agreement of long trajectories
with the authors' own code (no such code or printed trajectory exists here) -
"parity unpinned" for that single item.
"""
from __future__ import annotations

import numpy as np

STATE_O = 0  # Original  (bf16 row)
STATE_Q = 1  # Quantized (packed low-bit row)
STATE_E = 2  # Evicted

GROUP = 32   # channels per quantisation group

# Tuned constants the paper reports (Sec. V "Main Results").
PAPER_W = 32
PAPER_ALPHA = 0.75
PAPER_TAU = (7.774, 5.407, 5.528)
PAPER_GAMMA = 263.81


# --------------------------------------------------------------------------
# Sec. IV-C: observation-window attention and layer statistics
# --------------------------------------------------------------------------
def window_attention(q_win, k, scale, group):
    """Post-softmax attention of the last W prompt queries (eq. 2).

    q_win [Hq, W, d], k [Hkv, T, d] (values exactly representable in bf16),
    scale = softmax scale, group = Hq // Hkv (q-head h reads kv-head h // group).
    Window query i sits at absolute position T-W+i and sees keys j <= T-W+i
    (causal).  The softmax runs over the whole visible row; the slice to
    non-window keys is taken by the callers.  Returns a [Hq, W, T], zero where
    masked.
    """
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    Hq, W, d = q_win.shape
    Hkv, T, _ = k.shape
    assert Hq == Hkv * group and W <= T
    a = np.zeros((Hq, W, T), dtype=np.float64)
    for h in range(Hq):
        logits = scale * (q_win[h] @ k[h // group].T)          # [W, T]
        for i in range(W):
            nvis = T - W + i + 1
            row = logits[i, :nvis]
            e = np.exp(row - row.max())
            a[h, i, :nvis] = e / e.sum()
    return a


def window_lse(q_win, k, scale, group):
    """Natural-log normaliser of every window row of eq. 2: ln sum_{j <= T-W+i} exp(scale q_i.k_j), the
    per-row log-sum-exp that attention kernels return next to their output.  q_win [Hq, W, d], k [Hkv, T, d];
    returns [Hq, W] fp64."""
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    Hq, W, _ = q_win.shape
    T = k.shape[1]
    out = np.empty((Hq, W), dtype=np.float64)
    for h in range(Hq):
        logits = scale * (q_win[h] @ k[h // group].T)
        for i in range(W):
            row = logits[i, :T - W + i + 1]
            m = row.max()
            out[h, i] = m + np.log(np.exp(row - m).sum())
    return out


def layer_statistics(a, W):
    """Entropy, variance, kurtosis of the aggregated key distribution (eqs. 3-5).

    a [H, Wq, T] post-softmax attention of the window queries.  Only keys
    k < T - W enter.  p_k = (1/Z) sum_{h,q} a[h,q,k]; natural log;
    population moments over the n = T-W keys; kurtosis is the plain fourth
    standardised moment (no -3).  Reading for the degenerate case: if the
    variance is exactly 0 the kurtosis is reported as 0.
    Returns (H, V, Kurt, p).
    """
    a = np.asarray(a, dtype=np.float64)
    T = a.shape[2]
    n = T - W
    assert n >= 1
    c = a[:, :, :n].sum(axis=(0, 1))
    Z = c.sum()
    p = c / Z
    nz = p > 0
    H = -(p[nz] * np.log(p[nz])).sum()
    pbar = p.mean()
    dev = p - pbar
    m2 = (dev ** 2).mean()
    m4 = (dev ** 4).mean()
    kurt = m4 / (m2 * m2) if m2 > 0 else 0.0
    return float(H), float(m2), float(kurt), p


def prefill_accumulators(a, group):
    """First samples of the running per-token moments (eq. 9) from the window.

    For kv-head g and key j:  s1 = sum over the `group` q-heads of g and over the
    window queries that see j of a, s2 the same with a^2.  Masked entries are 0
    and add nothing.  Returns s1, s2 [Hkv, T].
    """
    a = np.asarray(a, dtype=np.float64)
    Hq, W, T = a.shape
    Hkv = Hq // group
    ag = a.reshape(Hkv, group, W, T)
    return ag.sum(axis=(1, 2)), (ag ** 2).sum(axis=(1, 2))


def sample_count(pos, P, T_prefill, W, group):
    """Number of (head, query) samples a token at `pos` has received once the
    query at position P has attended: group * (P - max(pos, T_prefill-W) + 1).
    Prompt tokens outside the window are first seen by the W window queries;
    later tokens by every query from their own position on."""
    pos = np.asarray(pos, dtype=np.int64)
    first = np.maximum(pos, T_prefill - W)
    return group * (P - first + 1)


def causal_attention_rows(q_rows, positions, k, v, scale, group):
    """Causal self-attention of selected prompt positions (the prefill pass the scorer can be fused into:
    the last W rows of this computation are exactly the rows of window_attention).

    q_rows [Hq, R, d] are the queries of absolute positions `positions` [R]; k, v [Hkv, T, d]; the query at
    position p sees keys j <= p.  Returns out [Hq, R, d] = softmax(scale * q k^T) v, fp64.
    """
    q_rows = np.asarray(q_rows, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    Hq, R, d = q_rows.shape
    out = np.zeros((Hq, R, d), dtype=np.float64)
    for h in range(Hq):
        g = h // group
        for r in range(R):
            nvis = int(positions[r]) + 1
            logits = scale * (k[g, :nvis] @ q_rows[h, r])
            e = np.exp(logits - logits.max())
            out[h, r] = (e / e.sum()) @ v[g, :nvis]
    return out


# --------------------------------------------------------------------------
# Sec. IV-D: OQ score, OQ ratio, per-layer budgets
# --------------------------------------------------------------------------
def oq_score(H, V, kurt, tau=PAPER_TAU):
    """q = H^(1/tau1) * V^(1/tau2) * Kurt^(1/tau3)  (eq. 6)."""
    return float(H) ** (1.0 / tau[0]) * float(V) ** (1.0 / tau[1]) * float(kurt) ** (1.0 / tau[2])


def oq_ratio(q):
    """rho_l = q_l / max_l q_l over the layers of one sequence (eq. 7).
    Reading: if every q is 0 (e.g. all-uniform attention) every rho is 1."""
    q = np.asarray(q, dtype=np.float64)
    mx = q.max()
    if not mx > 0:
        return np.ones_like(q)
    return q / mx


def row_bytes(d, bits):
    """(C_orig, C_quant) of eq. 1 for one token of one kv-head: bf16 K and V rows; packed K and V rows with
    their scales (grouped low-bit formats: fp16 scale and zero per 32 channels; fp8: one fp16 scale per row)."""
    c_q = 2 * (d + 2) if bits == 8 else 2 * (d * bits // 8 + (d // GROUP) * 4)
    return 4 * d, c_q


def budget_counts(rho, N, W, alpha=PAPER_ALPHA, every_step=False, byte_costs=None):
    """Token counts kept by a tailor (Alg. 1 'Assign origin budget', eq. 10).

    N = cache limit in tokens, same for every layer.  b = floor(alpha*(N-W))
    tokens survive outside the window (clamped to N-W-1 so that a tailor always
    frees a slot); of these n_o = min(floor(rho*(N-W)), b) are targeted
    Original and n_q = b - n_o Quantized.  every_step=True is the literal
    'at each step' reading of Sec. IV-F with no slack: the cache is kept full,
    b = N-W-1, so exactly one slot is freed and the tailor runs at every step.

    byte_costs=(C_orig, C_quant) reads eq. 1 and eq. 8 in bytes: the limit is
    N*C_orig bytes; the Original budget is n_o rows as above, and what the token
    rule would spend on Quantized rows at full cost, (b - n_o)*C_orig bytes, buys
    n_q = floor((b - n_o)*C_orig / C_quant) Quantized tokens instead.
    Returns (n_o, n_q, n_o + n_q).
    """
    b = N - W - 1 if every_step else int(np.floor(alpha * (N - W)))
    b = max(0, min(b, N - W - 1))
    n_o = min(int(np.floor(float(rho) * (N - W))), b)
    if byte_costs is not None:
        c_o, c_q = byte_costs
        n_q = ((b - n_o) * c_o) // c_q
        return n_o, n_q, n_o + n_q
    return n_o, b - n_o, b


# --------------------------------------------------------------------------
# Sec. IV-E: heavy-hitter score
# --------------------------------------------------------------------------
def hh_score(s1, s2, n, gamma=PAPER_GAMMA, exact32=False):
    """S = mu + gamma * var  with mu = s1/n, var = max(s2/n - mu^2, 0)  (eq. 9;
    reading: the quantity multiplied by gamma is the variance of the samples).

    exact32=True evaluates in IEEE fp32, one rounding per operation in exactly
    this order (div, div, mul, sub, max, mul, add): the precision in which the
    GPU path builds its selection keys.
    """
    if exact32:
        f = np.float32
        s1 = np.asarray(s1, dtype=f); s2 = np.asarray(s2, dtype=f)
        n = np.asarray(n).astype(f)
        mu = s1 / n
        ex2 = s2 / n
        var = np.maximum(ex2 - mu * mu, f(0))
        return mu + f(gamma) * var
    s1 = np.asarray(s1, dtype=np.float64); s2 = np.asarray(s2, dtype=np.float64)
    n = np.asarray(n, dtype=np.float64)
    mu = s1 / n
    var = np.maximum(s2 / n - mu * mu, 0.0)
    return mu + gamma * var


# --------------------------------------------------------------------------
# Sec. IV-F: tri-state tailor
# --------------------------------------------------------------------------
def selection_order(S, pos):
    """Indices sorted by (S descending, position ascending): the total order
    used for Top-b and Top-B_o (the paper does not say how ties break)."""
    S = np.asarray(S); pos = np.asarray(pos)
    return np.lexsort((pos, -S.astype(np.float64)))


def tailor_assign(S, pos, state, n_o, b):
    """New states of the eligible (non-window, live) tokens (eq. 10).

    rank < n_o -> target Original, n_o <= rank < b -> target Quantized,
    rank >= b -> Evicted.  Reading: states only move O -> Q -> E, a Quantized
    token is never promoted back (its bf16 row is gone), so new = max(old, target).
    Returns new_state (same order as the inputs).
    """
    S = np.asarray(S); pos = np.asarray(pos); state = np.asarray(state)
    order = selection_order(S, pos)
    rank = np.empty(len(S), dtype=np.int64)
    rank[order] = np.arange(len(S))
    target = np.where(rank < n_o, STATE_O, np.where(rank < b, STATE_Q, STATE_E))
    return np.maximum(state, target).astype(np.int8)


# --------------------------------------------------------------------------
# Low-bit quantiser (uniform, asymmetric, groups of 32 channels, fp16 scale/zero)
# --------------------------------------------------------------------------
def _f16_step(h, direction):
    """fp16 neighbour of every element of h towards -inf (direction=-1) or +inf (+1)."""
    h = np.asarray(h, dtype=np.float16)
    return np.nextafter(h, np.float16(direction * np.inf)).astype(np.float16)


def quantize_groups(x, bits):
    """Quantise groups of 32 channels, x [..., 32]; all arithmetic IEEE fp32,
    one rounding per operation, every group independent of the others.

    zero  = fp16(min), stepped one fp16 down where rounding put it above min;
    scale = fp16((max - zero) / qmax), stepped one fp16 up where the grid
            zero + qmax*scale would stop short of max;
    code  = clamp(rint((x - zero) / scale), 0, qmax), ties to even;
    a constant group (max == zero) gets scale 0 and codes 0.
    Returns (codes uint8[..., 32], scale fp16[...], zero fp16[...]).
    """
    f = np.float32
    x = np.asarray(x, dtype=f)
    assert x.shape[-1] == GROUP and np.all(np.isfinite(x)) and np.all(np.abs(x) <= 65504)
    qmax = f((1 << bits) - 1)
    mn = x.min(axis=-1); mx = x.max(axis=-1)
    zero_h = mn.astype(np.float16)
    zero_h = np.where(zero_h.astype(f) > mn, _f16_step(zero_h, -1), zero_h).astype(np.float16)
    z = zero_h.astype(f)
    r = (mx - z).astype(f)
    s = (r / qmax).astype(f)
    scale_h = s.astype(np.float16)
    short = (scale_h.astype(f) * qmax).astype(f) < r
    scale_h = np.where(short, _f16_step(scale_h, +1), scale_h).astype(np.float16)
    scale_h = np.where(r == 0, np.float16(0), scale_h).astype(np.float16)
    sc = scale_h.astype(f)
    safe = np.where(sc > 0, sc, f(1))
    t = ((x - z[..., None]).astype(f) / safe[..., None]).astype(f)
    codes = np.clip(np.rint(t), 0, qmax)
    codes = np.where((r == 0)[..., None], f(0), codes).astype(np.uint8)
    return codes, scale_h, zero_h


def quantize_row(x, bits):
    """Quantise one K or V row [d] group by group.  Returns codes uint8[d],
    scale fp16[d/32], zero fp16[d/32]."""
    x = np.asarray(x, dtype=np.float32)
    codes, scale, zero = quantize_groups(x.reshape(-1, GROUP), bits)
    return codes.reshape(-1), scale, zero


def dequantize_row(codes, scale, zero):
    """x~ = code * scale + zero per group, in fp64, not re-rounded to bf16."""
    codes = np.asarray(codes, dtype=np.float64)
    sc = np.repeat(np.asarray(scale, dtype=np.float64), GROUP)
    z = np.repeat(np.asarray(zero, dtype=np.float64), GROUP)
    return codes * sc + z


def pack_codes(codes, bits):
    """Canonical packing: little-endian fields inside a byte.  4-bit: byte k holds
    channel 2k in bits 0-3 and 2k+1 in bits 4-7; 2-bit: byte k holds channels
    4k..4k+3 in bits 0-1, 2-3, 4-5, 6-7."""
    codes = np.asarray(codes, dtype=np.uint8)
    per = 8 // bits
    c = codes.reshape(-1, per)
    out = np.zeros(c.shape[0], dtype=np.uint8)
    for i in range(per):
        out |= (c[:, i] << (bits * i)).astype(np.uint8)
    return out


def unpack_codes(packed, bits):
    packed = np.asarray(packed, dtype=np.uint8)
    per = 8 // bits
    mask = (1 << bits) - 1
    out = np.empty((packed.shape[0], per), dtype=np.uint8)
    for i in range(per):
        out[:, i] = (packed >> (bits * i)) & mask
    return out.reshape(-1)


# --------------------------------------------------------------------------
# fp8 quantiser with one scale per token row (Alg. 1 "Reconstruction Before
# Attention": x~ = q^ * s, "per-token scale"; Sec. V-C "fp8 form")
# --------------------------------------------------------------------------
# The paper does not say which 8-bit float it uses.  Reading taken: the OCP
# "E4M3" format without infinities (sign, 4 exponent bits with bias 7, 3
# mantissa bits; largest finite value 448; exponent field 0 holds subnormals
# m/8 * 2^-6; the all-ones magnitude 0x7F is NaN and never produced here).
E4M3_MAX = 448.0


def e4m3_magnitudes():
    """Value of every non-negative code 0..126, straight from the format's definition."""
    v = np.empty(127, dtype=np.float64)
    for code in range(127):
        e, m = code >> 3, code & 7
        v[code] = (m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return v


def quantize_fp8_rows(x):
    """Quantise rows x [..., d] (one K or V row of one token each); all arithmetic
    IEEE fp32, one rounding per operation.

    scale = fp16(amax / 448), stepped one fp16 up where 448*scale would stop short
            of amax = max|x| (so no element saturates); an all-zero row gets scale 0;
    t     = x / scale (fp32 division);
    code  = the E4M3 value nearest to |t| (a tie goes to the code with an even
            mantissa, i.e. the even code), capped at 448, sign bit set where x < 0.
    Returns (codes uint8[..., d], scale fp16[...]).
    """
    f = np.float32
    x = np.asarray(x, dtype=f)
    assert np.all(np.isfinite(x))
    amax = np.abs(x).max(axis=-1)
    s = (amax / f(E4M3_MAX)).astype(f)
    scale_h = s.astype(np.float16)
    short = (scale_h.astype(f) * f(E4M3_MAX)).astype(f) < amax
    scale_h = np.where(short, _f16_step(scale_h, +1), scale_h).astype(np.float16)
    scale_h = np.where(amax == 0, np.float16(0), scale_h).astype(np.float16)
    assert np.all(np.isfinite(scale_h.astype(f)))
    sc = scale_h.astype(f)
    safe = np.where(sc > 0, sc, f(1))
    t = np.abs((x / safe[..., None]).astype(f)).astype(np.float64)
    v = e4m3_magnitudes()
    mid = (v[:-1] + v[1:]) / 2.0                     # exact in fp64
    lo = np.searchsorted(mid, t, side="left")        # |t| <= mid[lo]  (first such), so v[lo] or a tie with v[lo+1]
    tie = (lo < len(mid)) & (t == mid[np.minimum(lo, len(mid) - 1)])
    code = np.where(tie & (lo % 2 == 1), lo + 1, lo)
    code = np.minimum(code, 126).astype(np.uint8)
    code = np.where((amax == 0)[..., None], np.uint8(0), code)
    code = np.where(x < 0, code | np.uint8(0x80), code).astype(np.uint8)
    return code, scale_h


def dequantize_fp8_row(codes, scale):
    """x~ = value(code) * scale in fp64, not re-rounded to bf16."""
    codes = np.asarray(codes, dtype=np.uint8)
    v = e4m3_magnitudes()[codes & 0x7F]
    return np.where(codes & 0x80, -v, v) * float(np.asarray(scale, dtype=np.float64).reshape(-1)[0])


# --------------------------------------------------------------------------
# Decode attention over a set of live tokens (plain definition)
# --------------------------------------------------------------------------
def attend(q, keys, values, scale):
    """softmax(scale * keys @ q) @ values for one head; returns (out[d], p[n])."""
    logits = scale * (np.asarray(keys, dtype=np.float64) @ np.asarray(q, dtype=np.float64))
    e = np.exp(logits - logits.max())
    p = e / e.sum()
    return p @ np.asarray(values, dtype=np.float64), p


# --------------------------------------------------------------------------
# Alg. 1 end to end, one (layer, sequence)
# --------------------------------------------------------------------------
class _Unit:
    """Live tokens of one kv-head, in arbitrary order."""

    def __init__(self, d):
        self.pos = np.zeros(0, dtype=np.int64)
        self.state = np.zeros(0, dtype=np.int8)
        self.kv = np.zeros((0, 2, d), dtype=np.float64)   # values attention sees (bf16 or dequantised)
        self.raw = np.zeros((0, 2, d), dtype=np.float32)  # bf16 rows (meaningful while Original)
        self.s1 = np.zeros(0, dtype=np.float64)
        self.s2 = np.zeros(0, dtype=np.float64)
        self.q = {}   # pos -> dict(k_codes, k_scale, k_zero, v_codes, v_scale, v_zero)


class SequenceCacheOracle:
    """The cache manager of Alg. 1 for one layer and one sequence.

    Every kv-head keeps its own scores, selection and token states (reading of
    'scores are averaged within each group to preserve KV sharing': the heads of
    a group are samples of one token's mean and variance).  Budgets are token
    counts; the tailor fires after the attention of the step at which the number
    of live tokens reaches N, so that the next append has room (byte_budget:
    see __init__).
    """

    def __init__(self, n_q_heads, n_kv_heads, head_dim, N, W=PAPER_W, alpha=PAPER_ALPHA,
                 gamma=PAPER_GAMMA, bits=4, every_step=False, byte_budget=False):
        self.every_step = every_step
        # byte_budget: the limit is N*C_orig bytes (eq. 1) and Quantized tokens are charged C_quant.  The
        # tailor still fires on a fixed schedule: occupancy is booked in rows as if every survivor of the
        # token rule's b were Original, which bounds the live bytes from above whatever the tokens' states.
        self.byte_budget = byte_budget
        self.occ = None        # booked occupancy in rows (== live tokens in token mode)
        self.Hq, self.Hkv, self.d = n_q_heads, n_kv_heads, head_dim
        self.G = n_q_heads // n_kv_heads
        self.N, self.W, self.alpha, self.gamma, self.bits = N, W, alpha, gamma, bits
        self.units = [_Unit(head_dim) for _ in range(n_kv_heads)]
        self.T = None          # prompt length
        self.P = None          # position of the latest token
        self.n_o = self.n_q = self.b = None
        self.n_tailors = 0
        self.last_tailor = None  # per kv-head dict(pos, S) of the eligible set of the latest tailor

    # ---- prefill ---------------------------------------------------------
    def commit(self, k, v, s1, s2, rho, S_override=None):
        """Load the prompt's K/V [Hkv, T, d] with window accumulators s1, s2 [Hkv, T]
        and the layer's OQ ratio; run the first tailor if the prompt already
        fills the cache (T >= N)."""
        k = np.asarray(k, dtype=np.float32); v = np.asarray(v, dtype=np.float32)
        T = k.shape[1]
        self.T, self.P = T, T - 1
        self.n_o, self.n_q, self.b = budget_counts(rho, self.N, self.W, self.alpha, self.every_step,
                                                   row_bytes(self.d, self.bits) if self.byte_budget else None)
        self.b_rows = budget_counts(rho, self.N, self.W, self.alpha, self.every_step)[2]
        self.occ = T
        for g, u in enumerate(self.units):
            u.pos = np.arange(T, dtype=np.int64)
            u.state = np.zeros(T, dtype=np.int8)
            u.raw = np.stack([k[g], v[g]], axis=1)
            u.kv = u.raw.astype(np.float64)
            u.s1 = np.asarray(s1[g], dtype=np.float64).copy()
            u.s2 = np.asarray(s2[g], dtype=np.float64).copy()
            u.q = {}
        if T >= self.N:
            self.tailor(S_override)

    # ---- decode ----------------------------------------------------------
    def decode_step(self, q, k_new, v_new, scale, S_override=None):
        """Append, attend, accumulate scores, tailor when full.
        q [Hq, d], k_new/v_new [Hkv, d].  Returns out [Hq, d] (fp64) and whether
        a tailor ran."""
        q = np.asarray(q, dtype=np.float64)
        k_new = np.asarray(k_new, dtype=np.float32); v_new = np.asarray(v_new, dtype=np.float32)
        self.P += 1
        out = np.empty((self.Hq, self.d), dtype=np.float64)
        for g, u in enumerate(self.units):
            assert self.occ < self.N
            row = np.stack([k_new[g], v_new[g]])[None]
            u.pos = np.append(u.pos, self.P)
            u.state = np.append(u.state, np.int8(STATE_O))
            u.raw = np.concatenate([u.raw, row], axis=0)
            u.kv = np.concatenate([u.kv, row.astype(np.float64)], axis=0)
            u.s1 = np.append(u.s1, 0.0); u.s2 = np.append(u.s2, 0.0)
            for hh in range(self.G):
                h = g * self.G + hh
                out[h], p = attend(q[h], u.kv[:, 0], u.kv[:, 1], scale)
                u.s1 += p
                u.s2 += p * p
        self.occ += 1
        fired = False
        if self.occ >= self.N:
            self.tailor(S_override)
            fired = True
        return out, fired

    # ---- tailor ----------------------------------------------------------
    def scores(self, g, exact32=False):
        u = self.units[g]
        n = sample_count(u.pos, self.P, self.T, self.W, self.G)
        return hh_score(u.s1, u.s2, n, self.gamma, exact32=exact32)

    def tailor(self, S_override=None):
        """Re-assign states of all tokens older than the W most recent positions.
        S_override: optional list (per kv-head) of dict pos -> fp32 score, used by
        lock-step parity tests so that both sides select on identical scores."""
        self.n_tailors += 1
        self.last_tailor = []
        window = min(self.W, self.P + 1)
        self.occ = window + min(self.b_rows, len(self.units[0].pos) - window)
        for g, u in enumerate(self.units):
            elig = u.pos < self.P + 1 - self.W
            idx = np.nonzero(elig)[0]
            if S_override is not None:
                S = np.array([S_override[g][int(p)] for p in u.pos[idx]], dtype=np.float32)
            else:
                S = self.scores(g)[idx]
            new_state = tailor_assign(S, u.pos[idx], u.state[idx], self.n_o, self.b)
            self.last_tailor.append({"pos": u.pos[idx].copy(), "S": np.asarray(S).copy(),
                                     "new_state": new_state.copy()})
            dem = idx[(new_state == STATE_Q) & (u.state[idx] == STATE_O)]
            if len(dem) and self.bits == 8:
                codes, sc = quantize_fp8_rows(u.raw[dem])          # [n, 2, d], [n, 2]
                none = np.zeros(1, dtype=np.float16)               # the format has no zero point
                for n_, j in enumerate(dem):
                    u.q[int(u.pos[j])] = dict(k_codes=codes[n_, 0], k_scale=sc[n_, 0:1], k_zero=none,
                                              v_codes=codes[n_, 1], v_scale=sc[n_, 1:2], v_zero=none)
                    u.kv[j, 0] = dequantize_fp8_row(codes[n_, 0], sc[n_, 0])
                    u.kv[j, 1] = dequantize_fp8_row(codes[n_, 1], sc[n_, 1])
                u.state[dem] = STATE_Q
            elif len(dem):
                d = self.d
                codes, sc, zr = quantize_groups(u.raw[dem].reshape(len(dem), 2, d // GROUP, GROUP),
                                                self.bits)
                codes = codes.reshape(len(dem), 2, d)
                for n_, j in enumerate(dem):
                    u.q[int(u.pos[j])] = dict(k_codes=codes[n_, 0], k_scale=sc[n_, 0], k_zero=zr[n_, 0],
                                              v_codes=codes[n_, 1], v_scale=sc[n_, 1], v_zero=zr[n_, 1])
                    u.kv[j, 0] = dequantize_row(codes[n_, 0], sc[n_, 0], zr[n_, 0])
                    u.kv[j, 1] = dequantize_row(codes[n_, 1], sc[n_, 1], zr[n_, 1])
                u.state[dem] = STATE_Q
            keep = np.ones(len(u.pos), dtype=bool)
            keep[idx[new_state == STATE_E]] = False
            for p in u.pos[~keep]:
                u.q.pop(int(p), None)
            u.pos, u.state, u.kv, u.raw = u.pos[keep], u.state[keep], u.kv[keep], u.raw[keep]
            u.s1, u.s2 = u.s1[keep], u.s2[keep]

    # ---- observability ---------------------------------------------------
    def counts(self, g):
        u = self.units[g]
        return int((u.state == STATE_O).sum()), int((u.state == STATE_Q).sum())

    def live_bytes(self, g):
        """eq. 1 cost of one kv-head: n_o*C_orig + n_q*C_quant with
        C_orig = 4d bytes (bf16 K and V), C_quant = 2*(d*bits/8 + (d/32)*4) for the
        grouped low-bit formats and 2*(d + 2) for fp8 rows with one fp16 scale."""
        no, nq = self.counts(g)
        co, cq = row_bytes(self.d, self.bits)
        return no * co + nq * cq
