// Tri-state tailor (Sec. IV-F eq. 10, Alg. 1 "KV Cache Tailor") and the prompt commit.
//
//   keys    : heavy-hitter score S = mu + gamma*var (eq. 9) -> 64-bit selection key
//             (fp32 bits of S) << 32 | (0xFFFFFFFF - position); larger key = better rank, so ties in
//             S go to the older token and the order is total.  0 marks "not eligible".
//   select  : exact k-th largest key by an 8-pass radix select, for k = n_o and k = b
//   plan    : classification of every slot and the lists that compact both pools in place
//   move    : quantise the demoted rows into free Q slots, fill holes with tail rows
//
// Everything that decides a state or a code is integer or single-rounded fp32 arithmetic in a fixed
// order (this file must be compiled with -ffp-contract=off).
#include <hip/hip_fp16.h>

#include "arkv_dev.h"

namespace arkv {

// ------------------------------------------------------------------------------------------
// score -> key
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float hh_score(float s1, float s2, int n, float gamma) {
  const float nf = (float)n;
  const float mu = s1 / nf;
  const float ex2 = s2 / nf;
  const float var = fmaxf(ex2 - mu * mu, 0.0f);
  return mu + gamma * var;
}

__device__ __forceinline__ uint64_t make_key(float S, int pos) {
  return ((uint64_t)__float_as_uint(S) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)pos);
}

template <int G>
__global__ __launch_bounds__(256) void k_tailor_keys(Pools P, TailorLaunch L) {
  const int gu = L.unit_begin + blockIdx.y;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= P.capO + P.capQ) return;
  const int2 cnt = P.cnt[gu];
  uint64_t key = 0;
  int pos = -1;
  float2 acc;
  if (i < P.capO) {
    if (i < cnt.x) { pos = P.opos[(size_t)gu * P.capO + i]; acc = P.oacc[(size_t)gu * P.capO + i]; }
  } else {
    const int j = i - P.capO;
    if (j < cnt.y) { pos = P.qpos[(size_t)gu * P.capQ + j]; acc = P.qacc[(size_t)gu * P.capQ + j]; }
  }
  if (pos >= 0 && pos < L.position + 1 - L.window) {
    const int first = pos > L.t_prefill - L.window ? pos : L.t_prefill - L.window;
    const int n = G * (L.position - first + 1);
    key = make_key(hh_score(acc.x, acc.y, n, L.gamma), pos);
  }
  P.keys[(size_t)gu * (P.capO + P.capQ) + i] = key;
}

__global__ __launch_bounds__(256) void k_commit_keys(uint64_t* keys, CommitLaunch L, int G) {
  const int lu = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= L.T) return;
  uint64_t key = 0;
  if (j < L.T - L.window) {
    const float2 a = L.pre[(size_t)lu * L.T + j];
    key = make_key(hh_score(a.x, a.y, G * L.window, L.gamma), j);
  }
  keys[(size_t)lu * L.T + j] = key;
}

// ------------------------------------------------------------------------------------------
// exact k-th largest key.  grid (2, units): x = 0 -> k = n_o[unit], x = 1 -> k = nb[unit].
// thr[unit][x] = that key, or ~0 when k = 0 (nothing qualifies).  k is clamped to the number of
// eligible keys, so "fewer candidates than b" keeps everything.
// ------------------------------------------------------------------------------------------
// Radix select, most significant byte first.  The candidates of a pass often share their byte (scores of
// one unit have the same exponent), which would serialise plain LDS atomics; lanes of a wave that hit the
// same bin as the wave's first candidate are therefore counted with a ballot and added once.  The keys a thread owns stay in registers
// for all passes when they fit (n <= 32 per thread), else they are re-read.  Keys are distinct (the position is part
// of them), so once the chosen bin holds a single candidate the remaining passes are skipped: its owner writes it.
constexpr int kSelKeys = 32;   // keys per thread held in registers
__global__ __launch_bounds__(1024) void k_select(const uint64_t* keys_all, size_t stride, int n,
                                                 const int32_t* n_o, const int32_t* nb, int unit_begin,
                                                 uint64_t* thr) {
  __shared__ int hist[256];
  __shared__ int s_sel, s_k, s_tot, s_cnt;
  const int lu = blockIdx.y, gu = unit_begin + lu, which = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const uint64_t* keys = keys_all + (size_t)lu * stride;
  const bool in_regs = n <= 1024 * kSelKeys;
  uint64_t mine[kSelKeys];
  if (in_regs) {
#pragma unroll
    for (int j = 0; j < kSelKeys; ++j) {
      const int i = tid + 1024 * j;
      mine[j] = i < n ? keys[i] : 0;
    }
  }
  int k = which == 0 ? n_o[gu] : nb[gu];
  uint64_t prefix = 0;
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    auto count = [&](uint64_t key) {
      bool cand = key != 0 && (pass == 0 || (key >> (shift + 8)) == prefix);
      const int bin = (int)((key >> shift) & 255);
      const unsigned long long todo = __ballot(cand);
      if (todo) {
        // the bin of the wave's first candidate is counted once for all lanes that share it (the common
        // case in the leading bytes); whoever differs adds for itself, to bins with little contention
        const int leader = __ffsll((long long)todo) - 1;
        const int lb = __shfl(bin, leader);
        const unsigned long long same = __ballot(cand && bin == lb);
        if (lane == leader) atomicAdd(&hist[lb], __popcll(same));
        else if (cand && bin != lb) atomicAdd(&hist[bin], 1);
      }
    };
    if (in_regs) {
#pragma unroll
      for (int j = 0; j < kSelKeys; ++j)
        if (1024 * j < n) count(mine[j]);               // uniform: whole rounds past the end are skipped
    } else {
      for (int i0 = 0; i0 < n; i0 += 1024) count(i0 + tid < n ? keys[i0 + tid] : 0);
    }
    __syncthreads();
    // wave 0: lane l owns bins 4l..4l+3; ge(bin) = candidates in bins >= bin
    if (tid < 64) {
      int h[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) h[i] = hist[4 * tid + i];
      const int own = h[0] + h[1] + h[2] + h[3];
      int above = own;                                   // inclusive suffix sum over lanes
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_down(above, o);
        if (tid + o < 64) above += t;
      }
      if (pass == 0 && tid == 0) s_tot = above;
      const int total = __shfl(above, 0);
      int kk = k;
      if (pass == 0 && kk > total) kk = total;           // fewer candidates than k: keep them all
      int ge = above - own;                              // candidates in bins of higher lanes
#pragma unroll
      for (int i = 3; i >= 0; --i) {
        const int gt = ge;
        ge += h[i];
        if (kk > 0 && gt < kk && kk <= ge) { s_sel = 4 * tid + i; s_k = kk - gt; s_cnt = h[i]; }
      }
    }
    __syncthreads();
    if (pass == 0) {
      if (k > s_tot) k = s_tot;
      if (k <= 0) {
        if (tid == 0) thr[(size_t)gu * 2 + which] = ~0ull;
        return;
      }
    }
    prefix = (prefix << 8) | (uint64_t)s_sel;
    k = s_k;
    const bool single = s_cnt == 1;                      // one candidate left: it is the answer
    __syncthreads();
    if (single && pass < 7) {
      auto claim = [&](uint64_t key) {
        if (key != 0 && (key >> shift) == prefix) thr[(size_t)gu * 2 + which] = key;
      };
      if (in_regs) {
#pragma unroll
        for (int j = 0; j < kSelKeys; ++j)
          if (1024 * j < n) claim(mine[j]);
      } else {
        for (int i0 = 0; i0 < n; i0 += 1024) claim(i0 + tid < n ? keys[i0 + tid] : 0);
      }
      return;
    }
  }
  if (tid == 0) thr[(size_t)gu * 2 + which] = prefix;
}

// ------------------------------------------------------------------------------------------
// block-wide exclusive scan of a packed counter (five 12-bit fields), 1024 threads
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t block_excl_scan(uint64_t v, uint64_t* sm /*[17]*/, uint64_t& total) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  uint64_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint64_t t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  if (lane == 63) sm[w] = inc;
  __syncthreads();
  if (tid == 0) {
    uint64_t run = 0;
    for (int i = 0; i < 16; ++i) { const uint64_t t = sm[i]; sm[i] = run; run += t; }
    sm[16] = run;
  }
  __syncthreads();
  const uint64_t res = sm[w] + inc - v;
  total = sm[16];
  __syncthreads();
  return res;
}

constexpr int F0 = 0, F1 = 12, F2 = 24, F3 = 36, F4 = 48;
__device__ __forceinline__ int fld(uint64_t v, int f) { return (int)((v >> f) & 0xFFFu); }

// ------------------------------------------------------------------------------------------
// in-place tailor plan.  One workgroup per unit.
//   plan: header | ohole[capO] | omov[capO] | dem[capO] | qfree[capQ] | qmov[capQ]
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_tailor_plan(Pools P, TailorLaunch L) {
  __shared__ uint64_t sm[17];
  __shared__ int tot[3];
  const int gu = L.unit_begin + blockIdx.x, tid = threadIdx.x;
  const int2 cnt = P.cnt[gu];
  const int cO = cnt.x, cQ = cnt.y;
  const uint64_t* keys = P.keys + (size_t)gu * (P.capO + P.capQ);
  const uint64_t thr_o = P.thr[(size_t)gu * 2], thr_b = P.thr[(size_t)gu * 2 + 1];
  int32_t* plan = P.plan + (size_t)gu * P.plan_stride;
  int32_t* ohole = plan + kPlanHdr;
  int32_t* omov = ohole + P.capO;
  int32_t* dem = omov + P.capO;
  int32_t* qfree = dem + P.capO;
  int32_t* qmov = qfree + P.capQ;

  // totals
  if (tid < 3) tot[tid] = 0;
  __syncthreads();
  int keepO = 0, nDem = 0, keepQ = 0, nElig = 0;
  for (int i = tid; i < cO; i += 1024) {
    const uint64_t k = keys[i];
    const bool keep = k == 0 || k >= thr_o;
    keepO += keep;
    nDem += (!keep && k >= thr_b);
    nElig += k != 0;
  }
  for (int i = tid; i < cQ; i += 1024) {
    const uint64_t k = keys[P.capO + i];
    keepQ += (k >= thr_b);
    nElig += 1;
  }
  for (int o = 32; o > 0; o >>= 1) {
    keepO += __shfl_xor(keepO, o); nDem += __shfl_xor(nDem, o); keepQ += __shfl_xor(keepQ, o);
  }
  if ((tid & 63) == 0) { atomicAdd(&tot[0], keepO); atomicAdd(&tot[1], nDem); atomicAdd(&tot[2], keepQ); }
  __syncthreads();
  const int cOn = tot[0], nD = tot[1], cQn = tot[2] + nD;

  // O pool lists
  int base_hole = 0, base_mov = 0, base_dem = 0;
  for (int c0 = 0; c0 < cO; c0 += 1024) {
    const int i = c0 + tid;
    bool hole = false, mov = false, d = false;
    if (i < cO) {
      const uint64_t k = keys[i];
      const bool keep = k == 0 || k >= thr_o;
      d = !keep && k >= thr_b;
      hole = i < cOn && !keep;
      mov = i >= cOn && keep;
    }
    const uint64_t v = ((uint64_t)hole << F0) | ((uint64_t)mov << F1) | ((uint64_t)d << F2);
    uint64_t total;
    const uint64_t ex = block_excl_scan(v, sm, total);
    if (hole) ohole[base_hole + fld(ex, F0)] = i;
    if (mov) omov[base_mov + fld(ex, F1)] = i;
    if (d) dem[base_dem + fld(ex, F2)] = i;
    base_hole += fld(total, F0); base_mov += fld(total, F1); base_dem += fld(total, F2);
  }
  // Q pool lists
  int base_free = 0, base_qmov = 0;
  const int qhi = cQ > cQn ? cQ : cQn;
  for (int c0 = 0; c0 < qhi; c0 += 1024) {
    const int i = c0 + tid;
    bool fr = false, mv = false;
    if (i < qhi) {
      const bool keep = i < cQ && keys[P.capO + i] >= thr_b;
      fr = i < cQn && !keep;
      mv = i >= cQn && keep;
    }
    const uint64_t v = ((uint64_t)fr << F3) | ((uint64_t)mv << F4);
    uint64_t total;
    const uint64_t ex = block_excl_scan(v, sm, total);
    if (fr) qfree[base_free + fld(ex, F3)] = i;
    if (mv) qmov[base_qmov + fld(ex, F4)] = i;
    base_free += fld(total, F3); base_qmov += fld(total, F4);
  }
  if (tid == 0) {
    plan[PL_CO_NEW] = cOn; plan[PL_CQ_NEW] = cQn; plan[PL_N_DEM] = nD;
    plan[PL_N_QMOV] = base_qmov; plan[PL_N_OMOV] = base_mov;
    plan[PL_CO_OLD] = cO; plan[PL_CQ_OLD] = cQ;
  }
}

// ------------------------------------------------------------------------------------------
// quantiser: one K or V row held by LPR lanes, 8 channels each (fp32 from bf16)
// ------------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dppf(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL,
                                                               0xf, 0xf, true));
}

__device__ __forceinline__ uint16_t f2h(float x) { return __half_as_ushort(__float2half_rn(x)); }
__device__ __forceinline__ float h2f(uint16_t h) { return __half2float(__ushort_as_half(h)); }
__device__ __forceinline__ uint16_t h_next_down(uint16_t h) {
  if ((h & 0x7fffu) == 0) return 0x8001u;
  return (h & 0x8000u) ? (uint16_t)(h + 1) : (uint16_t)(h - 1);
}
__device__ __forceinline__ uint16_t h_next_up(uint16_t h) {
  if ((h & 0x7fffu) == 0) return 0x0001u;
  return (h & 0x8000u) ? (uint16_t)(h - 1) : (uint16_t)(h + 1);
}

// x: the 8 channels of this lane; the 4 lanes of an aligned quad form one group of 32 channels.
// Returns the lane's packed codes (8*BITS bits) and the group's meta word (scale | zero << 16).
template <int BITS>
__device__ __forceinline__ void quantize8(const float (&x)[8], uint32_t& codes, uint32_t& meta) {
  const float qmax = (float)((1 << BITS) - 1);
  float mn = x[0], mx = x[0];
#pragma unroll
  for (int c = 1; c < 8; ++c) { mn = fminf(mn, x[c]); mx = fmaxf(mx, x[c]); }
  mn = fminf(mn, dppf<0xB1>(mn)); mx = fmaxf(mx, dppf<0xB1>(mx));
  mn = fminf(mn, dppf<0x4E>(mn)); mx = fmaxf(mx, dppf<0x4E>(mx));
  uint16_t zh = f2h(mn);
  float z = h2f(zh);
  if (z > mn) { zh = h_next_down(zh); z = h2f(zh); }
  const float r = mx - z;
  uint16_t sh = 0;
  codes = 0;
  if (r != 0.0f) {
    const float s = r / qmax;
    sh = f2h(s);
    float sc = h2f(sh);
    if (sc * qmax < r) { sh = h_next_up(sh); sc = h2f(sh); }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      float t = rintf((x[c] - z) / sc);
      t = fminf(fmaxf(t, 0.0f), qmax);
      codes |= (uint32_t)t << (BITS * c);
    }
  }
  meta = (uint32_t)sh | ((uint32_t)zh << 16);
}

__device__ __forceinline__ void unpack8(const uint4& r, float (&f)[8]) {
  f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
  f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
  f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
  f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
}

// fp8 rows with one scale per token (Alg. 1 "Reconstruction Before Attention": x~ = q^ * s).
// |t| <= 448 -> nearest E4M3 code (sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals below
// 2^-6, no infinities), ties to the even code, in integer arithmetic on the fp32 bits.
__device__ __forceinline__ uint32_t e4m3_code(float t) {
  const float a = fminf(fabsf(t), 448.0f);
  uint32_t code;
  if (a < 0.015625f) {
    code = (uint32_t)rintf(a * 512.0f);             // subnormals are multiples of 2^-9; 8 = the smallest normal
  } else {
    uint32_t b = __float_as_uint(a);
    b += 0x7FFFFu + ((b >> 20) & 1u);               // round to 3 mantissa bits, ties to even
    code = (((b >> 23) - 120u) << 3) | ((b >> 20) & 7u);
  }
  return code;
}

// x: the 8 channels of this lane; the LPR lanes of a row share one scale.
// Returns the lane's 8 codes (byte c = channel c) and the row's scale (fp16 bits).
template <int LPR>
__device__ __forceinline__ void quantize8_fp8(const float (&x)[8], uint2& codes, uint32_t& meta) {
  float amax = fabsf(x[0]);
#pragma unroll
  for (int c = 1; c < 8; ++c) amax = fmaxf(amax, fabsf(x[c]));
  amax = fmaxf(amax, dppf<0xB1>(amax));
  amax = fmaxf(amax, dppf<0x4E>(amax));
  amax = fmaxf(amax, dppf<0x141>(amax));             // 8 lanes
  if (LPR == 16) amax = fmaxf(amax, dppf<0x140>(amax));
  uint16_t sh = 0;
  codes = make_uint2(0, 0);
  if (amax != 0.0f) {
    const float s = amax / 448.0f;
    sh = f2h(s);
    float sc = h2f(sh);
    if (sc * 448.0f < amax) { sh = h_next_up(sh); sc = h2f(sh); }
    uint32_t w[2] = {0, 0};
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const uint32_t code = e4m3_code(x[c] / sc) | (x[c] < 0.0f ? 0x80u : 0u);
      w[c >> 2] |= code << (8 * (c & 3));
    }
    codes = make_uint2(w[0], w[1]);
  }
  meta = sh;
}

// One wave: lanes [0,LPR) quantise the K row, lanes [LPR,2LPR) the V row, into Q slot dst of unit gu.
template <int D, int BITS>
__device__ __forceinline__ void quantize_into(const Pools& P, int gu, int dst, const uint16_t* krow,
                                              const uint16_t* vrow, int lane) {
  constexpr int LPR = D / 8, CB = D * BITS / 8, NG = metas_per_row(D, BITS);
  const bool isv = lane >= LPR;
  const int sub = lane % LPR;
  // all 64 lanes run the arithmetic (the lane exchanges need them active); lanes >= 2LPR redo V
  const uint16_t* src = (isv ? vrow : krow) + sub * 8;
  const uint4 raw = *reinterpret_cast<const uint4*>(src);
  float x[8];
  unpack8(raw, x);
  // K: canonical row-major packing.  V: the same bytes, token-minor in blocks of kVBlock tokens (see Pools).
  uint8_t* cdst = P.qkc + ((size_t)gu * P.capQ + dst) * CB;
  uint32_t* mdst = P.qkm + ((size_t)gu * P.capQ + dst) * NG;
  uint8_t* vcu = P.qvc + (size_t)gu * P.capQv * CB;
  constexpr int MH = vmeta_per_row(D, BITS);
  uint16_t* vmu = P.qvm + (size_t)gu * P.capQv * MH;
  if constexpr (BITS == 8) {
    uint2 codes;
    uint32_t meta;
    quantize8_fp8<LPR>(x, codes, meta);
    if (lane < LPR) {
      *reinterpret_cast<uint2*>(cdst + ((sub & 3) * (D / 32) + (sub >> 2)) * 8) = codes;     // see kcode_index
      if (sub == 0) mdst[0] = meta;
    } else if (lane < 2 * LPR) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        vcu[vcode_index(dst, 8 * sub + i, CB, BITS)] = (uint8_t)((i < 4 ? codes.x >> (8 * i) : codes.y >> (8 * (i - 4))) & 0xffu);
      if (sub == 0) vmu[vmeta_index(dst, 0, MH)] = (uint16_t)meta;
    }
  } else {
    uint32_t codes, meta;
    quantize8<BITS>(x, codes, meta);
    if (lane < LPR) {
      const int chunk = (sub & 3) * (D / 32) + (sub >> 2);                                   // see kcode_index
      if (BITS == 4) *reinterpret_cast<uint32_t*>(cdst + chunk * 4) = codes;
      else *reinterpret_cast<uint16_t*>(cdst + chunk * 2) = (uint16_t)codes;
      if ((sub & 3) == 0) mdst[sub >> 2] = meta;
    } else if (lane < 2 * LPR) {
#pragma unroll
      for (int i = 0; i < BITS; ++i) vcu[vcode_index(dst, BITS * sub + i, CB, BITS)] = (uint8_t)((codes >> (8 * i)) & 0xffu);
      if ((sub & 3) == 0) {
        vmu[vmeta_index(dst, sub >> 2, MH)] = (uint16_t)(meta & 0xffffu);              // scale
        vmu[vmeta_index(dst, D / kGroup + (sub >> 2), MH)] = (uint16_t)(meta >> 16);   // zero point
      }
    }
  }
}

template <int D, int BITS>
__global__ __launch_bounds__(256) void k_tailor_move_q(Pools P, TailorLaunch L) {
  constexpr int CB = D * BITS / 8, NG = metas_per_row(D, BITS);
  const int gu = L.unit_begin + blockIdx.y, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int32_t* plan = P.plan + (size_t)gu * P.plan_stride;
  const int nD = plan[PL_N_DEM], nM = plan[PL_N_QMOV];
  const int32_t* dem = plan + kPlanHdr + 2 * P.capO;
  const int32_t* qfree = dem + P.capO;
  const int32_t* qmov = qfree + P.capQ;
  for (int item = blockIdx.x * 4 + w; item < nD + nM; item += gridDim.x * 4) {
    const int dst = qfree[item];
    if (item < nD) {
      const int src = dem[item];
      const size_t o = (size_t)gu * P.capO + src;
      quantize_into<D, BITS>(P, gu, dst, P.ok + o * D, P.ov + o * D, lane);
      if (lane == 0) {
        P.qpos[(size_t)gu * P.capQ + dst] = P.opos[o];
        P.qacc[(size_t)gu * P.capQ + dst] = P.oacc[o];
      }
    } else {
      const int src = qmov[item - nD];
      const size_t so = (size_t)gu * P.capQ + src, d_ = (size_t)gu * P.capQ + dst;
      // K: code bytes, 4 per lane; V: one byte column per lane (token-minor blocks)
      for (int b = lane * 4; b < CB; b += 256)
        *reinterpret_cast<uint32_t*>(P.qkc + d_ * CB + b) = *reinterpret_cast<const uint32_t*>(P.qkc + so * CB + b);
      uint8_t* vcu = P.qvc + (size_t)gu * P.capQv * CB;
      for (int b = lane; b < CB; b += 64) vcu[vcode_index(dst, b, CB, BITS)] = vcu[vcode_index(src, b, CB, BITS)];
      constexpr int MH = vmeta_per_row(D, BITS);
      uint16_t* vmu = P.qvm + (size_t)gu * P.capQv * MH;
      if (lane < MH) vmu[vmeta_index(dst, lane, MH)] = vmu[vmeta_index(src, lane, MH)];
      if (lane < NG) P.qkm[d_ * NG + lane] = P.qkm[so * NG + lane];
      if (lane == 0) { P.qpos[d_] = P.qpos[so]; P.qacc[d_] = P.qacc[so]; }
    }
  }
}

template <int D>
__global__ __launch_bounds__(256) void k_tailor_move_o(Pools P, TailorLaunch L) {
  constexpr int LPR = D / 8;
  const int gu = L.unit_begin + blockIdx.y, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int32_t* plan = P.plan + (size_t)gu * P.plan_stride;
  const int nM = plan[PL_N_OMOV];
  const int32_t* ohole = plan + kPlanHdr;
  const int32_t* omov = ohole + P.capO;
  for (int item = blockIdx.x * 4 + w; item < nM; item += gridDim.x * 4) {
    const size_t so = (size_t)gu * P.capO + omov[item], d_ = (size_t)gu * P.capO + ohole[item];
    if (lane < 2 * LPR) {
      uint16_t* base = lane < LPR ? P.ok : P.ov;
      const int sub = lane % LPR;
      *reinterpret_cast<uint4*>(base + d_ * D + sub * 8) = *reinterpret_cast<const uint4*>(base + so * D + sub * 8);
    }
    if (lane == 0) { P.opos[d_] = P.opos[so]; P.oacc[d_] = P.oacc[so]; }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) P.cnt[gu] = make_int2(plan[PL_CO_NEW], plan[PL_CQ_NEW]);
}

// ------------------------------------------------------------------------------------------
// prompt commit: classification of prompt positions and scatter into the empty pools
//   plan: header | osrc[capO] | qsrc[capQ]
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_commit_plan(Pools P, CommitLaunch L, const uint64_t* keys_all) {
  __shared__ uint64_t sm[17];
  const int lu = blockIdx.x, gu = L.unit_begin + lu, tid = threadIdx.x;
  const uint64_t* keys = keys_all + (size_t)lu * L.T;
  const uint64_t thr_o = P.thr[(size_t)gu * 2], thr_b = P.thr[(size_t)gu * 2 + 1];
  int32_t* plan = P.plan + (size_t)gu * P.plan_stride;
  int32_t* osrc = plan + kPlanHdr;
  int32_t* qsrc = osrc + P.capO;
  int bo = 0, bq = 0;
  // eight consecutive positions per thread and round: one block scan per 8192 positions (the two counts are
  // carried in the halves of one 64-bit word), positions stay in ascending order
  constexpr int E = 8;
  for (int c0 = 0; c0 < L.T; c0 += 1024 * E) {
    const int j0 = c0 + E * tid;
    unsigned om = 0, qm = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if (j0 + e < L.T) {
        const uint64_t k = keys[j0 + e];
        const bool o = k == 0 || k >= thr_o;          // key 0 = window position
        om |= (unsigned)o << e;
        qm |= (unsigned)(!o && k >= thr_b) << e;
      }
    }
    const uint64_t v = (uint64_t)__popc(om) | ((uint64_t)__popc(qm) << 32);
    uint64_t total;
    const uint64_t ex = block_excl_scan(v, sm, total);
    int io = bo + (int)(ex & 0xFFFFFFFFu), iq = bq + (int)(ex >> 32);
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if ((om >> e) & 1u) osrc[io++] = j0 + e;
      if ((qm >> e) & 1u) qsrc[iq++] = j0 + e;
    }
    bo += (int)(total & 0xFFFFFFFFu); bq += (int)(total >> 32);
  }
  if (tid == 0) { plan[PL_CO_NEW] = bo; plan[PL_CQ_NEW] = bq; P.cnt[gu] = make_int2(bo, bq); }
}

template <int D, int BITS>
__global__ __launch_bounds__(256) void k_commit_scatter(Pools P, CommitLaunch L) {
  constexpr int LPR = D / 8;
  const int lu = blockIdx.y, gu = L.unit_begin + lu, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int32_t* plan = P.plan + (size_t)gu * P.plan_stride;
  const int32_t* osrc = plan + kPlanHdr;
  const int32_t* qsrc = osrc + P.capO;
  const int cO = L.select ? plan[PL_CO_NEW] : L.T, cQ = L.select ? plan[PL_CQ_NEW] : 0;
  const uint16_t* K = L.k + (size_t)lu * L.T * D;
  const uint16_t* V = L.v + (size_t)lu * L.T * D;
  const float2* pre = L.pre + (size_t)lu * L.T;
  for (int item = blockIdx.x * 4 + w; item < cO + cQ; item += gridDim.x * 4) {
    if (item < cO) {
      const int j = L.select ? osrc[item] : item;
      const size_t d_ = (size_t)gu * P.capO + item;
      if (lane < 2 * LPR) {
        const uint16_t* src = lane < LPR ? K : V;
        uint16_t* dst = lane < LPR ? P.ok : P.ov;
        const int sub = lane % LPR;
        *reinterpret_cast<uint4*>(dst + d_ * D + sub * 8) = *reinterpret_cast<const uint4*>(src + (size_t)j * D + sub * 8);
      }
      if (lane == 0) { P.opos[d_] = j; P.oacc[d_] = pre[j]; }
    } else {
      const int dst = item - cO, j = qsrc[dst];
      quantize_into<D, BITS>(P, gu, dst, K + (size_t)j * D, V + (size_t)j * D, lane);
      if (lane == 0) { P.qpos[(size_t)gu * P.capQ + dst] = j; P.qacc[(size_t)gu * P.capQ + dst] = pre[j]; }
    }
  }
  if (!L.select && blockIdx.x == 0 && threadIdx.x == 0) P.cnt[gu] = make_int2(L.T, 0);
}

// ------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------
static int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

template <int D, int BITS>
static void launch_tailor_moves(const Pools& P, const TailorLaunch& a, hipStream_t s) {
  dim3 gq(clampi((P.capQ + 3) / 4, 1, 256), a.n_units), go(clampi((P.capO + 3) / 4, 1, 256), a.n_units);
  hipLaunchKernelGGL((k_tailor_move_q<D, BITS>), gq, dim3(256), 0, s, P, a);
  hipLaunchKernelGGL((k_tailor_move_o<D>), go, dim3(256), 0, s, P, a);
}

hipError_t launch_tailor(const Pools& P, const TailorLaunch& a, hipStream_t s) {
  if (a.n_pending > 0) {
    hipError_t e = launch_flush_scores(P, a.unit_begin, a.n_units, a.n_pending, a.slot, s);
    if (e != hipSuccess) return e;
  }
  const int ntot = P.capO + P.capQ;
  dim3 gk((ntot + 255) / 256, a.n_units);
  switch (P.G) {
    case 1: hipLaunchKernelGGL((k_tailor_keys<1>), gk, dim3(256), 0, s, P, a); break;
    case 2: hipLaunchKernelGGL((k_tailor_keys<2>), gk, dim3(256), 0, s, P, a); break;
    case 4: hipLaunchKernelGGL((k_tailor_keys<4>), gk, dim3(256), 0, s, P, a); break;
    case 8: hipLaunchKernelGGL((k_tailor_keys<8>), gk, dim3(256), 0, s, P, a); break;
    default: return hipErrorInvalidValue;
  }
  hipLaunchKernelGGL(k_select, dim3(2, a.n_units), dim3(1024), 0, s,
                     P.keys + (size_t)a.unit_begin * ntot, (size_t)ntot, ntot, P.n_o, P.nb, a.unit_begin, P.thr);
  hipLaunchKernelGGL(k_tailor_plan, dim3(a.n_units), dim3(1024), 0, s, P, a);
  if (P.D == 128 && P.bits == 4) launch_tailor_moves<128, 4>(P, a, s);
  else if (P.D == 128 && P.bits == 2) launch_tailor_moves<128, 2>(P, a, s);
  else if (P.D == 64 && P.bits == 4) launch_tailor_moves<64, 4>(P, a, s);
  else if (P.D == 64 && P.bits == 2) launch_tailor_moves<64, 2>(P, a, s);
  else if (P.D == 128 && P.bits == 8) launch_tailor_moves<128, 8>(P, a, s);
  else if (P.D == 64 && P.bits == 8) launch_tailor_moves<64, 8>(P, a, s);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

template <int D, int BITS>
static void launch_commit_scatter(const Pools& P, const CommitLaunch& a, hipStream_t s) {
  dim3 g(clampi((P.capO + P.capQ + 3) / 4, 1, 1024), a.n_units);
  hipLaunchKernelGGL((k_commit_scatter<D, BITS>), g, dim3(256), 0, s, P, a);
}

// The layer's budgets (per sequence: Original target and survivor count) reach the device as launch
// arguments, so that the commit stays ordered on the caller's stream without a staging buffer.
struct BudgetArgs { int n_o[64], nb[64]; };
__global__ void k_set_budgets(int32_t* n_o, int32_t* nb, int unit_begin, int hkv, int seq0, int n_seq, BudgetArgs a) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_seq * hkv) return;
  const int u = unit_begin + seq0 * hkv + i;
  n_o[u] = a.n_o[i / hkv];
  nb[u] = a.nb[i / hkv];
}

hipError_t launch_set_budgets(const Pools& P, int unit_begin, int hkv, int batch, const int32_t* n_o_seq,
                              const int32_t* nb_seq, hipStream_t s) {
  for (int s0 = 0; s0 < batch; s0 += 64) {
    const int n = batch - s0 < 64 ? batch - s0 : 64;
    BudgetArgs a;
    for (int i = 0; i < n; ++i) { a.n_o[i] = n_o_seq[s0 + i]; a.nb[i] = nb_seq[s0 + i]; }
    for (int i = n; i < 64; ++i) { a.n_o[i] = 0; a.nb[i] = 0; }
    hipLaunchKernelGGL(k_set_budgets, dim3((n * hkv + 255) / 256), dim3(256), 0, s, P.n_o, P.nb, unit_begin, hkv, s0, n, a);
  }
  return hipGetLastError();
}

hipError_t launch_commit(const Pools& P, const CommitLaunch& a, uint64_t* ckeys, hipStream_t s) {
  if (a.select) {
    hipLaunchKernelGGL(k_commit_keys, dim3((a.T + 255) / 256, a.n_units), dim3(256), 0, s, ckeys, a, P.G);
    hipLaunchKernelGGL(k_select, dim3(2, a.n_units), dim3(1024), 0, s, (const uint64_t*)ckeys, (size_t)a.T,
                       a.T, P.n_o, P.nb, a.unit_begin, P.thr);
    hipLaunchKernelGGL(k_commit_plan, dim3(a.n_units), dim3(1024), 0, s, P, a, (const uint64_t*)ckeys);
  }
  if (P.D == 128 && P.bits == 4) launch_commit_scatter<128, 4>(P, a, s);
  else if (P.D == 128 && P.bits == 2) launch_commit_scatter<128, 2>(P, a, s);
  else if (P.D == 64 && P.bits == 4) launch_commit_scatter<64, 4>(P, a, s);
  else if (P.D == 64 && P.bits == 2) launch_commit_scatter<64, 2>(P, a, s);
  else if (P.D == 128 && P.bits == 8) launch_commit_scatter<128, 8>(P, a, s);
  else if (P.D == 64 && P.bits == 8) launch_commit_scatter<64, 8>(P, a, s);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace arkv
