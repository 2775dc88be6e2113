// Decode step kernels (Alg. 1 "Decoding Phase" + "Reconstruction Before Attention", fused):
//   k_decode_attend : append + split-K attention of one query per head over the bf16 pool and the
//                     packed pool (dequantisation inside the QK and PV loops)
//                     + the merge of the split-K partials by the unit's last workgroup (partials
//                     move through device-scope atomics, see st_dev2; a device-scope fence per
//                     workgroup instead was measured 3-6x slower, a second kernel costs a launch gap
//                     per step)
//                     + on every (kRing-1)-th launch the score update (Eq. 9) of the steps since the
//                     last one: a step's probabilities need its final softmax denominator, which
//                     only exists after the merge, so they are formed later, from the step's stored
//                     query against the key tile that is in registers anyway (same instructions on
//                     the same bits as the step itself), several waiting steps per MFMA operand.
//                     The other launches only read the cache.
//   k_flush_scores  : the same score update on its own, when something needs the scores now
//                     (tailor, export)
#include <hip/hip_fp16.h>

#include "arkv.h"
#include "arkv_dev.h"

namespace arkv {

constexpr float kNegBig = -1.0e30f;

// 2^x as one v_exp_f32 (arguments here are bounded above and may be hugely negative -> 0)
__device__ __forceinline__ float fexp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL,
                                                               0xf, 0xf, true));
}

// DPP controls: 0xB1 quad_perm [1,0,3,2], 0x4E quad_perm [2,3,0,1], 0x141 row_half_mirror, 0x140 row_mirror.
// Applied in this order they reduce over the 16 lanes of a DPP row and leave the result in every lane.
__device__ __forceinline__ float row_sum16(float x) {
  x += dpp_mov<0xB1>(x);
  x += dpp_mov<0x4E>(x);
  x += dpp_mov<0x141>(x);
  x += dpp_mov<0x140>(x);
  return x;
}
__device__ __forceinline__ float row_max16(float x) {
  x = fmaxf(x, dpp_mov<0xB1>(x));
  x = fmaxf(x, dpp_mov<0x4E>(x));
  x = fmaxf(x, dpp_mov<0x141>(x));
  x = fmaxf(x, dpp_mov<0x140>(x));
  return x;
}

// over the whole wave, same result in every lane, fixed order
__device__ __forceinline__ float lane_value(float x, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), l));
}
__device__ __forceinline__ float wave_max(float x) {
  x = row_max16(x);
  return fmaxf(fmaxf(lane_value(x, 0), lane_value(x, 16)), fmaxf(lane_value(x, 32), lane_value(x, 48)));
}
__device__ __forceinline__ float wave_sum(float x) {
  x = row_sum16(x);
  return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}

__device__ __forceinline__ void unpack_bf16x8(const uint4& r, float (&f)[8]) {
  f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
  f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
  f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
  f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
}

__device__ __forceinline__ float half_bits_to_float(uint32_t h) {
  return __half2float(__ushort_as_half((unsigned short)(h & 0xffffu)));
}

__device__ __forceinline__ uint16_t float_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Rows [ao,bo) of the O pool and [aq,bq) of the Q pool that split s of S owns.  Rows are weighted by
// their measured cost (bf16 row = 16 units, packed row = wq units) so that splits take equal time; the
// last split also appends the new token, which is charged like kNewTokenRows bf16 rows.
// The two divisions (by S and by wq) are multiplications by reciprocals that the host puts in the launch
// arguments: the cut points come first in every workgroup's life, in front of its first request to HBM.  They
// need not be exact quotients, only the same monotone function of s everywhere, 0 at s = 0 and everything at S.
constexpr unsigned kNewTokenRows = 32;
__host__ __device__ inline unsigned mulhi_u32(unsigned a, unsigned b) {
  return (unsigned)(((unsigned long long)a * (unsigned long long)b) >> 32);
}
__host__ __device__ inline void split_range(int cO, int cQ, int wq, int S, int s, SplitRecip rc, int& ao, int& bo,
                                            int& aq, int& bq) {
  // tot * S fits 32 bits: the library only creates caches with 16 (capO + capQ + 32) * 128 < 2^32
  const unsigned tot = 16u * (unsigned)cO + (unsigned)wq * (unsigned)cQ + 16u * kNewTokenRows;
  auto cut = [&](int i) {
    if (i <= 0) return 0u;
    if (i >= S) return tot;
    const unsigned v = mulhi_u32(tot * (unsigned)i, rc.inv_s);
    return v < tot ? v : tot;
  };
  const unsigned v0 = cut(s), v1 = cut(s + 1);
  auto mapO = [&](unsigned v) { const int r = (int)((v + 15u) / 16u); return r < cO ? r : cO; };
  auto mapQ = [&](unsigned v) {
    if (v <= 16u * (unsigned)cO) return 0;
    const unsigned x = v - 16u * (unsigned)cO + (unsigned)wq - 1u;
    int r = (int)(wq > 1 ? mulhi_u32(x, rc.inv_wq) : x);
    r = (r + kVBlock - 1) & ~(kVBlock - 1);      // packed rows are dealt in whole value blocks
    return r < cQ ? r : cQ;
  };
  ao = mapO(v0); bo = mapO(v1); aq = mapQ(v0); bq = mapQ(v1);
}

// 8 packed codes -> 8 bf16 values 128 + code, element order [c0,c4,c1,c5,c2,c6,c3,c7]
// (bf16 0x4300 is 128.0 with a 7-bit mantissa, so OR-ing a code < 128 into it adds the code exactly).
template <int BITS>
__device__ __forceinline__ uint4 codes_to_bf16_biased(uint32_t cw) {
  uint4 r;
  if (BITS == 4) {
    r.x = (cw & 0x000F000Fu) | 0x43004300u;
    r.y = ((cw >> 4) & 0x000F000Fu) | 0x43004300u;
    r.z = ((cw >> 8) & 0x000F000Fu) | 0x43004300u;
    r.w = ((cw >> 12) & 0x000F000Fu) | 0x43004300u;
  } else {
    const uint32_t y = (cw & 0xFFu) | ((cw & 0xFF00u) << 8);
    r.x = (y & 0x00030003u) | 0x43004300u;
    r.y = ((y >> 2) & 0x00030003u) | 0x43004300u;
    r.z = ((y >> 4) & 0x00030003u) | 0x43004300u;
    r.w = ((y >> 6) & 0x00030003u) | 0x43004300u;
  }
  return r;
}

// bf16 pairs (c0,c1)(c2,c3)(c4,c5)(c6,c7) -> (c0,c4)(c1,c5)(c2,c6)(c3,c7)
__device__ __forceinline__ uint4 permute_for_codes(const uint4& q) {
  uint4 r;
  r.x = (q.x & 0xFFFFu) | (q.z << 16);
  r.y = (q.x >> 16) | (q.z & 0xFFFF0000u);
  r.z = (q.y & 0xFFFFu) | (q.w << 16);
  r.w = (q.y >> 16) | (q.w & 0xFFFF0000u);
  return r;
}

// D[m][n] += sum_k A[m][k] B[k][n], 16x16x32 bf16.  Lane l holds A[l%16][8(l/16)..+7],
// B[8(l/16)..+7][l%16] and D[4(l/16)..+3][l%16].
__device__ __forceinline__ f32x4 mfma16(const uint4& a, const uint4& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// ---- pieces shared by the attention kernel and the stand-alone score update ----------------------

// Query operand of a unit: lane holds head lane%16 (zero beyond G), channels 32kk + 8(lane/16) .. +7.
template <int D, int G>
__device__ __forceinline__ void load_query(const uint16_t* q_unit, int lane, uint4 (&qa)[D / 32]) {
  const int tok = lane & 15, blk = lane >> 4;
  const uint16_t* q = q_unit + (size_t)(tok < G ? tok : 0) * D + 8 * blk;
#pragma unroll
  for (int kk = 0; kk < D / 32; ++kk) {
    const uint4 v = *reinterpret_cast<const uint4*>(q + 32 * kk);
    qa[kk] = tok < G ? v : make_uint4(0, 0, 0, 0);
  }
}

// Dot products of the unit's heads with 16 bf16 key rows held in operand layout.
template <int KK>
__device__ __forceinline__ f32x4 dots_bf16(const uint4 (&qa)[KK], const uint4 (&kb)[KK]) {
  f32x4 C = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) C = mfma16(qa[kk], kb[kk], C);
  return C;
}

// ---- packed row formats -------------------------------------------------------------------------
// PackedFmt<D, HPL, BITS> gives the attention loop what it needs of a Quantized row: what to keep of a
// query, how lane (token lane%16, block lane/16) loads the key codes of row rk and turns them into the
// token's HPL dot products (one 16-byte load per lane: a row's key chunks are stored [lane block][k-step]).
// Values are ValueFmt's business, further down.
//
// BITS = 2, 4: uniform codes, groups of 32 channels, fp16 scale and zero per group.  Codes are OR-ed into
// bf16 "128 + code" operands, one MFMA per group; scale, zero and the 128 offset are applied to the
// per-group results, which needs the query's per-group channel sums (an MFMA against an all-ones tile).
template <int D, int HPL, int BITS>
struct PackedFmt {
  static constexpr int KK = D / 32, CB = D * BITS / 8, NG = D / kGroup, CW = BITS;
  struct Query { uint4 qp[KK]; float qs[KK][HPL]; };
  struct Keys { uint32_t cw[KK], meta[KK]; };
  static __device__ __forceinline__ void prep(const uint4 (&qa)[KK], Query& q) {
    const uint4 ones = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      f32x4 C = {0.f, 0.f, 0.f, 0.f};
      C = mfma16(qa[kk], ones, C);
#pragma unroll
      for (int i = 0; i < HPL; ++i) q.qs[kk][i] = C[i];
      q.qp[kk] = permute_for_codes(qa[kk]);
    }
  }
  static __device__ __forceinline__ void load_keys(const uint8_t* kc, const uint32_t* km, int rk, int blk, Keys& k) {
    // the KK chunks this lane block needs of the row are contiguous (kcode_index): one load; so are the row's
    // KK metadata words
    const uint8_t* p = kc + (unsigned)rk * CB + blk * (KK * CW);
    uint32_t raw[4] = {0, 0, 0, 0};
    if constexpr (KK * CW == 16) { const uint4 v = *reinterpret_cast<const uint4*>(p); raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w; }
    else if constexpr (KK * CW == 8) { const uint2 v = *reinterpret_cast<const uint2*>(p); raw[0] = v.x; raw[1] = v.y; }
    else raw[0] = *reinterpret_cast<const uint32_t*>(p);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      k.cw[kk] = BITS == 4 ? raw[kk] : ((raw[kk >> 1] >> (16 * (kk & 1))) & 0xFFFFu);
    const uint32_t* m = km + (unsigned)rk * NG;
    if constexpr (KK == 4) { const uint4 v = *reinterpret_cast<const uint4*>(m); k.meta[0] = v.x; k.meta[1] = v.y; k.meta[2] = v.z; k.meta[3] = v.w; }
    else { const uint2 v = *reinterpret_cast<const uint2*>(m); k.meta[0] = v.x; k.meta[1] = v.y; }
  }
  static __device__ __forceinline__ void dots(const Query& q, const Keys& k, float (&x)[HPL]) {
#pragma unroll
    for (int i = 0; i < HPL; ++i) x[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      f32x4 C = {0.f, 0.f, 0.f, 0.f};
      C = mfma16(q.qp[kk], codes_to_bf16_biased<BITS>(k.cw[kk]), C);
      // sum_c q_c (sc code_c + z) = sc (C - 128 qs) + z qs = sc C + (z - 128 sc) qs
      const float sc = half_bits_to_float(k.meta[kk]), z = half_bits_to_float(k.meta[kk] >> 16);
      const float zz = fmaf(-128.0f, sc, z);
#pragma unroll
      for (int i = 0; i < HPL; ++i) x[i] = fmaf(sc, C[i], fmaf(zz, q.qs[kk][i], x[i]));
    }
  }
  // the same against a round of waiting steps, whose prepared operand rows (qp) and channel sums (qs) sit in LDS
  static __device__ __forceinline__ void dots_pending(const uint16_t (*qp)[D + 8], const float (*qs)[16], const Keys& k, int tok,
                                                      int blk, float (&x)[HPL]) {
#pragma unroll
    for (int i = 0; i < HPL; ++i) x[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const uint4 q = *reinterpret_cast<const uint4*>(&qp[tok][32 * kk + 8 * blk]);
      const float4 s4 = *reinterpret_cast<const float4*>(&qs[kk][4 * blk]);
      const float s[4] = {s4.x, s4.y, s4.z, s4.w};
      f32x4 C = {0.f, 0.f, 0.f, 0.f};
      C = mfma16(q, codes_to_bf16_biased<BITS>(k.cw[kk]), C);
      const float sc = half_bits_to_float(k.meta[kk]), z = half_bits_to_float(k.meta[kk] >> 16);
      const float zz = fmaf(-128.0f, sc, z);
#pragma unroll
      for (int i = 0; i < HPL; ++i) x[i] = fmaf(sc, C[i], fmaf(zz, s[i], x[i]));
    }
  }
};

// BITS = 8: the paper's own format (Alg. 1 "Reconstruction Before Attention", x~ = q^ * s): one fp8 E4M3
// byte per channel and one fp16 scale per row.  Every E4M3 value is a bf16 value, so the codes become MFMA
// operands by conversion alone and the row scale multiplies the finished dot product.
__device__ __forceinline__ void fp8x8_to_f32(const uint2& w, float (&f)[8]) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, true);
  const f32x2 c = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, true);
  f[0] = a[0]; f[1] = a[1]; f[2] = b[0]; f[3] = b[1]; f[4] = c[0]; f[5] = c[1]; f[6] = d[0]; f[7] = d[1];
}
__device__ __forceinline__ uint4 fp8x8_to_bf16x8(const uint2& w) {
  float f[8];
  fp8x8_to_f32(w, f);
  uint4 r;   // exact: an E4M3 value has 4 significant bits
  r.x = (__float_as_uint(f[0]) >> 16) | (__float_as_uint(f[1]) & 0xffff0000u);
  r.y = (__float_as_uint(f[2]) >> 16) | (__float_as_uint(f[3]) & 0xffff0000u);
  r.z = (__float_as_uint(f[4]) >> 16) | (__float_as_uint(f[5]) & 0xffff0000u);
  r.w = (__float_as_uint(f[6]) >> 16) | (__float_as_uint(f[7]) & 0xffff0000u);
  return r;
}
template <int D, int HPL>
struct PackedFmt<D, HPL, 8> {
  static constexpr int KK = D / 32, CB = D, NG = 1;
  struct Query { uint4 q[KK]; };
  struct Keys { uint2 cw[KK]; uint32_t meta; };
  static __device__ __forceinline__ void prep(const uint4 (&qa)[KK], Query& q) {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) q.q[kk] = qa[kk];
  }
  static __device__ __forceinline__ void load_keys(const uint8_t* kc, const uint32_t* km, int rk, int blk, Keys& k) {
    const uint4* p = reinterpret_cast<const uint4*>(kc + (unsigned)rk * CB + blk * (KK * 8));   // see kcode_index
#pragma unroll
    for (int h = 0; h < KK / 2; ++h) {
      const uint4 v = p[h];
      k.cw[2 * h] = make_uint2(v.x, v.y);
      k.cw[2 * h + 1] = make_uint2(v.z, v.w);
    }
    k.meta = km[rk];
  }
  static __device__ __forceinline__ void dots(const Query& q, const Keys& k, float (&x)[HPL]) {
    f32x4 C = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) C = mfma16(q.q[kk], fp8x8_to_bf16x8(k.cw[kk]), C);
    const float sc = half_bits_to_float(k.meta);
#pragma unroll
    for (int i = 0; i < HPL; ++i) x[i] = C[i] * sc;
  }
};

// ---- packed value rows on the matrix cores --------------------------------------------------------
// PV contracts over tokens, so the value codes are stored token-minor (Pools::qvc): lane (n = lane%16,
// kb = lane/16) of a 16x16x32 fp16 MFMA reads 8 bytes = one byte column of tokens 8kb..8kb+7 of a 32-token
// block and turns them into the B operand of output channel(s) of that column.  The A operand is the
// probabilities of the block times the tokens' scales of the channel group, rounded to fp16
// (lane = head lane%16, tokens 8kb..+7).  Codes enter as fp16 "1024 + code * 2^s" (0x6400 OR-ed with the
// masked byte: exact, no shift, no conversion); the offset is taken out again with the sum of the A operand
// (an MFMA against all ones), the factor 2^s at the end, and the zero points come from one more MFMA of
// the plain probabilities against the tokens' zero points (one column per group; a column of ones gives
// the probabilities' sum, i.e. the softmax denominator, in the same rounding as the numerator).
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ f32x4 mfma16h(const uint4& a, const uint4& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ uint4 mul_f16x8(const uint4& a, const uint4& b) {
  return __builtin_bit_cast(uint4, __builtin_bit_cast(f16x8, a) * __builtin_bit_cast(f16x8, b));
}
// bytes (b0, b1, b2, b3) of x -> fp16 pairs (0x6400 | b0, 0x6400 | b1), (0x6400 | b2, 0x6400 | b3)
__device__ __forceinline__ void bytes_to_f16_biased(uint32_t x, uint32_t& lo, uint32_t& hi) {
  lo = __builtin_amdgcn_perm(0x64646464u, x, 0x04010400u);
  hi = __builtin_amdgcn_perm(0x64646464u, x, 0x04030402u);
}
constexpr uint32_t kOnesF16 = 0x3C003C00u;

template <int D, int BITS>
struct ValueFmt {
  static constexpr int CB = D * BITS / 8;            // byte columns of a row
  static constexpr int NG = D / kGroup;              // scale groups
  static constexpr int MH = vmeta_per_row(D, BITS);
  static constexpr int NACC = D / 16;                // PV MFMAs (accumulators of 16 channels) per block
  static constexpr int APG = NACC / NG;              // accumulators per group (2)
  static constexpr int NLD = BITS == 4 ? CB / 16 : NG;   // 8-byte code loads per lane and block
  static constexpr int ZCOLS = NG;                   // columns of the correction MFMA that hold zero points
  static constexpr bool kBiased = true;
  // The A operand has 16 rows and a unit only G heads, so one operand carries several groups: rows
  // [r * RPG, r * RPG + G) hold the probabilities times the scales of the operand's r-th group, and the PV
  // MFMAs of that group find their results in those rows.
  template <int G> static constexpr int rpg() { return G <= 4 ? 4 : 8; }          // operand rows per group
  template <int G> static constexpr int gpa() { return 16 / rpg<G>(); }           // groups per A operand
  template <int G> static constexpr int na() { return (NG + gpa<G>() - 1) / gpa<G>(); }   // A operands per block
  static constexpr int NSC = 2;                      // >= na<G>() for every G
  struct Blk { uint2 cw[NLD]; uint4 sc[NSC]; uint4 z; };
  // gs[j]: the group whose scales this lane's row of A operand j needs
  static __device__ __forceinline__ void load(const uint8_t* vc, const uint16_t* vm, int b32, int n, int kb,
                                              const int (&gs)[NSC], int nsc, Blk& b) {
    // the lane's NLD byte columns x 8 tokens are contiguous (vcode_index)
    constexpr int NL = BITS == 2 ? 8 : 16;
    const uint4* base = reinterpret_cast<const uint4*>(vc + (size_t)b32 * (CB * kVBlock) + (size_t)((kb * NL + (n & (NL - 1))) * NLD) * 8);
#pragma unroll
    for (int i = 0; i < NLD / 2; ++i) {
      const uint4 v = base[i];
      b.cw[2 * i] = make_uint2(v.x, v.y);
      b.cw[2 * i + 1] = make_uint2(v.z, v.w);
    }
    const uint16_t* mb = vm + (size_t)b32 * (MH * kVBlock) + 8 * kb;
#pragma unroll
    for (int j = 0; j < NSC; ++j)
      if (j < nsc) b.sc[j] = *reinterpret_cast<const uint4*>(mb + gs[j] * kVBlock);
    const uint4 zl = *reinterpret_cast<const uint4*>(mb + (NG + (n < NG ? n : NG - 1)) * kVBlock);
    const uint32_t fill = n == NG ? kOnesF16 : 0u;
    b.z = n < NG ? zl : make_uint4(fill, fill, fill, fill);
  }
  static __device__ __forceinline__ int group_of(int a) { return a / APG; }
  // B operand of accumulator a
  static __device__ __forceinline__ uint4 operand(const Blk& b, int a, int n) {
    uint32_t mask;
    uint2 w;
    if constexpr (BITS == 4) {
      w = b.cw[a >> 1];
      mask = (a & 1) ? 0xF0F0F0F0u : 0x0F0F0F0Fu;
    } else {
      w = b.cw[a >> 1];
      const uint32_t m0 = n < 8 ? 0x03030303u : 0x0C0C0C0Cu;
      mask = (a & 1) ? m0 << 4 : m0;
    }
    uint4 r;
    bytes_to_f16_biased(w.x & mask, r.x, r.y);
    bytes_to_f16_biased(w.y & mask, r.z, r.w);
    return r;
  }
  // what the accumulator holds is 2^s times the channel's sum: its reciprocal
  static __device__ __forceinline__ float unscale(int a, int n) {
    if constexpr (BITS == 4) return (a & 1) ? 0.0625f : 1.0f;
    else return (a & 1) ? (n < 8 ? 0.0625f : 0.015625f) : (n < 8 ? 1.0f : 0.25f);
  }
  static __device__ __forceinline__ int channel(int a, int n) {
    if constexpr (BITS == 4) return 2 * (16 * (a >> 1) + n) + (a & 1);
    else return 4 * (8 * (a >> 1) + (n & 7)) + 2 * (a & 1) + (n >> 3);
  }
};

// fp8 rows: one byte per channel, one scale per row; E4M3 values are fp16 values, so no offset and no zero point.
template <int D>
struct ValueFmt<D, 8> {
  static constexpr int CB = D, NG = 1, MH = 1, NACC = D / 16, APG = NACC, NLD = D / 16, ZCOLS = 0;
  static constexpr bool kBiased = false;
  template <int G> static constexpr int rpg() { return 16; }     // one scale per row: the operand's rows are the heads
  template <int G> static constexpr int gpa() { return 1; }
  template <int G> static constexpr int na() { return 1; }
  static constexpr int NSC = 1;
  struct Blk { uint2 cw[NLD]; uint4 sc[1]; uint4 z; };
  static __device__ __forceinline__ void load(const uint8_t* vc, const uint16_t* vm, int b32, int n, int kb,
                                              const int (&)[NSC], int, Blk& b) {
    const uint4* base = reinterpret_cast<const uint4*>(vc + (size_t)b32 * (CB * kVBlock) + (size_t)((kb * 16 + n) * NLD) * 8);
#pragma unroll
    for (int i = 0; i < NLD / 2; ++i) {
      const uint4 v = base[i];
      b.cw[2 * i] = make_uint2(v.x, v.y);
      b.cw[2 * i + 1] = make_uint2(v.z, v.w);
    }
    b.sc[0] = *reinterpret_cast<const uint4*>(vm + (size_t)b32 * kVBlock + 8 * kb);
    const uint32_t fill = n == 0 ? kOnesF16 : 0u;
    b.z = make_uint4(fill, fill, fill, fill);
  }
  static __device__ __forceinline__ int group_of(int) { return 0; }
  static __device__ __forceinline__ uint4 operand(const Blk& b, int a, int) {
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    const uint2 w = b.cw[a];
    uint4 r;
    r.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((int)w.x, 1.0f, false));
    r.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((int)w.x, 1.0f, true));
    r.z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((int)w.y, 1.0f, false));
    r.w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((int)w.y, 1.0f, true));
    return r;
  }
  static __device__ __forceinline__ float unscale(int, int) { return 1.0f; }
  static __device__ __forceinline__ int channel(int a, int n) { return 16 * a + n; }
};

// Eq. 9 running moments: the lane's HPL logits of one token (base-2 units) -> probabilities with the
// step's final (max, 1/sum) -> their sum and sum of squares over the unit's heads, valid in block 0.
template <int HPL, int HB>
__device__ __forceinline__ float2 prob_moments(const float (&x)[HPL], const float (&pm)[HPL], const float (&pinv)[HPL]) {
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int i = 0; i < HPL; ++i) {
    const float p = fexp2(x[i] - pm[i]) * pinv[i];
    s1 += p;
    s2 = fmaf(p, p, s2);
  }
  if constexpr (HB == 2) { s1 += __shfl_xor(s1, 16); s2 += __shfl_xor(s2, 16); }
  return make_float2(s1, s2);
}

// ---- score update of the steps that wait for it -------------------------------------------------
// Per unit the latest steps' queries, scales and final softmax constants sit in a ring (Pools::qprev,
// qscale, fin).  A workgroup that is to add n waiting steps to (s1, s2) first copies their state to LDS;
// then, per 16-token key tile, the logits of every waiting step are recomputed (same MFMA sequence on the
// same bits as in the step itself), turned into probabilities and their moments added in step order.
// The MFMA has 16 query rows and a step only needs G of them, so several waiting steps share one operand
// ("round"): step r * SPR + b occupies rows [b * RPS, b * RPS + G) of round r's operand; rows nothing fills are zero.
template <int G> struct PendingShape {
  static constexpr int RPS = G <= 4 ? 4 : 8;                       // operand rows per step
  static constexpr int SPR = 16 / RPS;                             // steps per round
  static constexpr int ROUNDS = (kRing - 1 + SPR - 1) / SPR;       // 2 (G <= 4) or 4 (G = 8)
};
template <int D, int G>
struct PendingLds {
  // index ROUNDS of qp / qs: the query of the step in flight (rows 0 .. G-1), so that launches that update the
  // scores need not hold its packed-format operands in registers
  // Row pitch D + 8 elements (2D + 16 bytes): the 16 rows that the lanes of a quarter wave read as 16-byte
  // vectors then fall into 16 different bank groups; at a pitch of 2D bytes they all fall into the same one
  static constexpr int PITCH = D + 8;
  uint16_t q[PendingShape<G>::ROUNDS][16][PITCH];        // round r's operand rows (bf16)
  uint16_t qp[PendingShape<G>::ROUNDS + 1][16][PITCH];   // the same rows as the grouped packed formats want them (permute_for_codes)
  float qs[PendingShape<G>::ROUNDS + 1][D / 32][16]; // ... and each row's channel sums per group of 32
  float2 fin[kRing - 1][G];                      // a waiting step's final (max, 1/sum) per head
  float scale[kRing - 1];                        // its softmax scale * log2(e)
};

// All 256 threads of the workgroup; ends with a barrier.  packed: also prepare qp / qs, a round per wave; q_now (may be
// null): this step's query rows [G][D], prepared as index ROUNDS.
template <int D, int G>
__device__ __forceinline__ void stage_pending(const Pools& P, int gu, int n, int slot, PendingLds<D, G>& sm, int tid,
                                              bool packed, const uint16_t* q_now = nullptr) {
  constexpr int nthreads = 256;                  // both callers run 256-thread workgroups
  using PS = PendingShape<G>;
  constexpr int KK = D / 32;
  const size_t LU = P.fin_stride / G;
  // every load is requested before the first store: one at a time, each would cost a memory round trip in front
  // of the tile loop (the loop below has at most kStageBatch iterations per thread for 256 threads)
  constexpr int NQ = PS::ROUNDS * 16 * (D / 8);
  constexpr int kStageBatch = (NQ + 255) / 256;
  uint4 qv[kStageBatch];
#pragma unroll
  for (int b = 0; b < kStageBatch; ++b) {
    const int i = tid + b * nthreads;
    const int row = i / (D / 8), c = i % (D / 8);            // row = 16 r + operand row
    const int step = (row / 16) * PS::SPR + (row % 16) / PS::RPS, head = (row % 16) % PS::RPS;
    qv[b] = make_uint4(0, 0, 0, 0);
    if (i < NQ && head < G && step < n) {
      const int sl = (slot - n + step + kRing) % kRing;
      qv[b] = reinterpret_cast<const uint4*>(P.qprev + ((size_t)sl * P.fin_stride + (size_t)gu * G + head) * D)[c];
    }
  }
  float2 fv = make_float2(0.f, 0.f);
  float sv = 0.f;
  if (tid < n * G) {                                            // n * G <= 8 * 8 < 256
    const int j = tid / G, h = tid % G;
    const int sl = (slot - n + j + kRing) % kRing;
    fv = P.fin[(size_t)sl * P.fin_stride + (size_t)gu * G + h];
    if (h == 0) sv = P.qscale[(size_t)sl * LU + gu];
  }
#pragma unroll
  for (int b = 0; b < kStageBatch; ++b) {
    const int i = tid + b * nthreads;
    if (i < NQ) *reinterpret_cast<uint4*>(&sm.q[i / (16 * (D / 8))][(i / (D / 8)) % 16][8 * (i % (D / 8))]) = qv[b];
  }
  if (tid < n * G) {
    const int j = tid / G, h = tid % G;
    sm.fin[j][h] = fv;
    if (h == 0) sm.scale[j] = sv;
  }
  __syncthreads();
  if (packed) {
    const int lane = tid & 63, tok = lane & 15, blk = lane >> 4;
    const uint4 ones = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
    for (int r = tid >> 6; r < PS::ROUNDS + (q_now ? 1 : 0); r += nthreads >> 6) {
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        uint4 qo;
        if (r < PS::ROUNDS) {
          qo = *reinterpret_cast<const uint4*>(&sm.q[r][tok][32 * kk + 8 * blk]);
        } else {
          const uint4 v = *reinterpret_cast<const uint4*>(q_now + (size_t)(tok < G ? tok : 0) * D + 32 * kk + 8 * blk);
          qo = tok < G ? v : make_uint4(0, 0, 0, 0);
        }
        f32x4 C = {0.f, 0.f, 0.f, 0.f};
        C = mfma16(qo, ones, C);                      // every column: the rows' sums over this group's channels
        *reinterpret_cast<uint4*>(&sm.qp[r][tok][32 * kk + 8 * blk]) = permute_for_codes(qo);
        if (tok == 0) *reinterpret_cast<float4*>(&sm.qs[r][kk][4 * blk]) = make_float4(C[0], C[1], C[2], C[3]);
      }
    }
    __syncthreads();
  }
}

// Adds the moments of the n waiting steps to (s1, s2) of the lane's token.  dots(r, qop, x) must fill x with
// the token's raw dot products against round r's query operand (qop: the plain bf16 rows); a token takes part
// from waiting step `first` on (it did not exist before).  The result is valid in lanes of block 0.
//
// The logits of the steps of a round land in different lane blocks, where the probabilities and moments of up
// to four steps are computed by the same instructions; block 0 then collects them and adds them in step
// order (the same fp32 additions as one step at a time).
template <int D, int G, typename Dots>
__device__ __forceinline__ float2 fold_pending(const PendingLds<D, G>& sm, int n, int first, float2 ac, int lane, Dots&& dots) {
  constexpr int KK = D / 32, HB = (G + 3) / 4, HPL = G < 4 ? G : 4;
  constexpr int RPS = PendingShape<G>::RPS, SPR = PendingShape<G>::SPR;
  const int tok = lane & 15, blk = lane >> 4;
  for (int j0 = 0; j0 < n; j0 += SPR) {
    uint4 qop[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qop[kk] = *reinterpret_cast<const uint4*>(&sm.q[j0 / SPR][tok][32 * kk + 8 * blk]);
    float x[HPL], pm[HPL], pinv[HPL];
    dots(j0 / SPR, qop, x);
    // this lane's results are rows 4*blk .. +3 of the operand: step js, heads h0 .. h0+3
    const int js = min(j0 + (4 * blk) / RPS, n - 1), h0 = (4 * blk) % RPS;
    const float sc = sm.scale[js];
#pragma unroll
    for (int i = 0; i < HPL; ++i) {
      const float2 f = sm.fin[js][h0 + i];
      pm[i] = f.x; pinv[i] = f.y;
      x[i] *= sc;
    }
    const float2 m = prob_moments<HPL, HB>(x, pm, pinv);   // valid in the first block of every step
#pragma unroll
    for (int b = 0; b < SPR; ++b) {
      const int srcl = tok + 16 * (b * RPS / 4);
      const float mx = __shfl(m.x, srcl), my = __shfl(m.y, srcl);
      const int j = j0 + b;
      if (j < n && j >= first) { ac.x += mx; ac.y += my; }
    }
  }
  return ac;
}

// Profiling builds (-DARKV_PHASE_TRACE, which also turns on the merge's own marks) record a 100 MHz timestamp
// per workgroup at the phase boundaries marked TRACE(i) / TRACE_M(i); arkv_debug_phase_trace copies them out.
// Product builds compile none of it.
#ifdef ARKV_PHASE_TRACE
#define ARKV_PHASE_TRACE_MERGE
__device__ unsigned long long g_trace[8192][8];
#define TRACE(i) do { if (threadIdx.x == 0) g_trace[blockIdx.y * gridDim.x + blockIdx.x][i] = wall_clock64(); } while (0)
// word 7 of a workgroup's row: the XCC_ID hardware register (id 20, all 32 bits; the XCD number is its low 4 bits)
#define TRACE_XCD() do { if (threadIdx.x == 0) g_trace[blockIdx.y * gridDim.x + blockIdx.x][7] = \
    (unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20); } while (0)
__global__ void k_trace_mark(int slot) { if (threadIdx.x == 0) g_trace[8190][slot] = wall_clock64(); }
#else
#define TRACE(i)
#define TRACE_XCD()
#endif
#ifdef ARKV_PHASE_TRACE_MERGE
__device__ unsigned long long g_trace_m[8192][8];
#define TRACE_M(i) do { if (threadIdx.x == 0) g_trace_m[blockIdx.y * gridDim.x + blockIdx.x][i] = wall_clock64(); } while (0)
#else
#define TRACE_M(i)
#endif

// Split-K partials cross workgroups that may sit on different XCDs, whose L2 caches are not coherent
// with each other for ordinary accesses.  They are therefore written and read with device-scope relaxed
// atomics (write-through stores, loads that do not hit a stale L2 line); no cache-wide flush is needed.
// What this rests on is the AMDGPU backend's documented memory model for the gfx942 family, which gfx950
// belongs to: an agent-scope atomic store or load is a global access with sc1 set, which writes through to /
// is served from the level at which the whole device is coherent, and an agent-scope read-modify-write is
// performed at that level.  A release at agent scope is, by the same table, an L2 write-back followed by
// s_waitcnt vmcnt(0), and an acquire an L2 invalidate; the write-back and the invalidate exist for data that
// ordinary stores left dirty in, or ordinary loads pulled into, an XCD's L2.  Nothing the merge consumes is
// written or read by ordinary accesses, so only the wait remains: a wave's partial stores are acknowledged
// (s_waitcnt 0) before the workgroup's barrier, and the ticket is taken after the barrier.
// (two adjacent floats, 8-byte aligned, per access)
__device__ __forceinline__ void st_dev2(float* p, float a, float b) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p),
                     (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_dev2(const float* p) {
  return __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Merge of a unit's split-K partials by the workgroup that finished last: output row, the step's
// (max, 1/sum) per head, token count.  All 256 threads of that workgroup take part; a thread owns pairs of
// adjacent channels (8-byte loads), and the partials of up to 64 splits are requested before the first is
// used, so the merge costs one round trip to memory where a launch has many splits per unit.
template <int D, int G>
__device__ __forceinline__ void combine_splits(const Pools& P, const DecodeLaunch& L, int lu, int gu, int tid) {
  __shared__ __align__(16) float cw[G][kMaxSplits];   // weight of split s for head h; 0 beyond the launch's splits
  __shared__ float cInv[G];
  constexpr int RS = G * (D + 2);                  // floats per split
  constexpr int NP = G * D / 2;                    // channel pairs per split
  constexpr int NI = (NP + 255) / 256;             // pairs per thread
  constexpr int NB = (G <= 2 ? 32 : 64) / NI;      // splits per batch of loads (NI * NB * 2 registers)
  TRACE_M(0);
  const float* part = P.part + (size_t)(gu - L.part_unit0) * P.max_splits * RS;
  const int S = L.splits;
  int hh[NI], off[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int idx = min(tid + 256 * i, NP - 1);
    hh[i] = idx / (D / 2);
    off[i] = hh[i] * (D + 2) + 2 * (idx % (D / 2));
  }
  unsigned long long v[NI][NB];
  auto load_batch = [&](int s0) {
#pragma unroll
    for (int g = 0; g < NB / 16; ++g) {
      if (s0 + 16 * g < S) {                       // uniform: whole groups of 16 splits are skipped
#pragma unroll
        for (int jj = 0; jj < 16; ++jj)
#pragma unroll
          for (int i = 0; i < NI; ++i)
            v[i][16 * g + jj] = ld_dev2(part + (size_t)min(s0 + 16 * g + jj, S - 1) * RS + off[i]);
      }
    }
  };
  // (max, sum) of the splits: wave w takes heads w and w + 4; a lane takes splits lane and lane + 64 and the
  // wave reduces in a fixed order.  The pairs are requested first and the first batch of partial values right
  // behind them, so that the weights are worked out while the values are on their way: one round trip.
  {
    constexpr int NH = (G + 3) / 4;
    const int lane = tid & 63, w = tid >> 6;
    float m0[NH], l0[NH], m1[NH], l1[NH];
#pragma unroll
    for (int k = 0; k < NH; ++k) {
      const int h = min(w + 4 * k, G - 1);
      m0[k] = m1[k] = kNegBig; l0[k] = l1[k] = 0.f;
      if (lane < S) {
        const unsigned long long ml = ld_dev2(part + (size_t)lane * RS + h * (D + 2) + D);
        m0[k] = __uint_as_float((unsigned)ml); l0[k] = __uint_as_float((unsigned)(ml >> 32));
      }
      if (lane + 64 < S) {
        const unsigned long long ml = ld_dev2(part + (size_t)(lane + 64) * RS + h * (D + 2) + D);
        m1[k] = __uint_as_float((unsigned)ml); l1[k] = __uint_as_float((unsigned)(ml >> 32));
      }
    }
    load_batch(0);
    TRACE_M(1);
#pragma unroll
    for (int k = 0; k < NH; ++k) {
      const int h = w + 4 * k;
      if (h < G) {                                 // uniform per wave
        const float M = wave_max(fmaxf(m0[k], m1[k]));
        const float w0 = lane < S ? exp2f(m0[k] - M) : 0.f, w1 = lane + 64 < S ? exp2f(m1[k] - M) : 0.f;
        cw[h][lane] = w0;
        cw[h][lane + 64] = w1;
        const float l = wave_sum(fmaf(l0[k], w0, l1[k] * w1));
        if (lane == 0) {
          cInv[h] = 1.0f / l;
          P.fin[(size_t)L.slot * P.fin_stride + (size_t)gu * G + h] = make_float2(M, 1.0f / l);
        }
      }
    }
  }
  TRACE_M(2);
  __syncthreads();
  TRACE_M(3);
  float o[NI][2];
#pragma unroll
  for (int i = 0; i < NI; ++i) o[i][0] = o[i][1] = 0.f;
  for (int s0 = 0;;) {
#pragma unroll
    for (int g = 0; g < NB / 16; ++g) {
      if (s0 + 16 * g < S) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
          for (int i = 0; i < NI; ++i) {
            const float4 w4 = *reinterpret_cast<const float4*>(&cw[hh[i]][s0 + 16 * g + 4 * q]);
            const float wgt[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const unsigned long long x = v[i][16 * g + 4 * q + e];
              o[i][0] = fmaf(__uint_as_float((unsigned)x), wgt[e], o[i][0]);
              o[i][1] = fmaf(__uint_as_float((unsigned)(x >> 32)), wgt[e], o[i][1]);
            }
          }
        }
      }
    }
    s0 += NB;
    if (s0 >= S) break;
    load_batch(s0);
  }
  TRACE_M(4);
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int idx = tid + 256 * i;
    if (idx < NP) {
      const float r0 = o[i][0] * cInv[hh[i]], r1 = o[i][1] * cInv[hh[i]];
      *reinterpret_cast<float2*>(P.outf + (size_t)gu * G * D + 2 * idx) = make_float2(r0, r1);
      *reinterpret_cast<uint32_t*>(L.out + (size_t)lu * G * D + 2 * idx) =
          (uint32_t)float_to_bf16_rne(r0) | ((uint32_t)float_to_bf16_rne(r1) << 16);
    }
  }
  if (tid == 0) P.cnt[gu].x += 1;
  TRACE_M(5);
}

// Attention of one query per head over this split's share of a unit's cache.
//
// A wave works on tiles of 16 tokens.  QK^T of a tile is D/32 MFMAs (A = the unit's G query rows padded
// to 16, B = 16 key rows loaded from HBM straight into operand layout); lane (token t = lane%16, block
// b = lane/16) then owns the logits of token t for heads 4b..4b+3.  FOLD launches multiply the same key
// tile with the waiting steps' queries as well (fold_pending) and update the tokens' (s1, s2).  This
// step's probabilities go through a small LDS buffer to the value layout (lane = 8 channels of one of
// 64/(D/8) rows), where PV of the bf16 rows runs on the vector ALU (HBM-bound as it is); packed rows take
// PV to the matrix cores (ValueFmt).  The softmax reference maximum is only moved when a logit of a bf16
// row exceeds it by more than 8 (base-2 units), which is rare, so the accumulators are almost never rescaled.
// What a workgroup needs before it can request its first tile, packed together at the front of the launch
// arguments so that it arrives in one round trip of the scalar cache (copies of fields of Pools / DecodeLaunch).
struct DecodeHot {
  const uint16_t* ok; const uint16_t* ov; float2* oacc; float2* qacc; const uint16_t* q;
  size_t fin_stride;
  int capO, capQ, splits, wq, known, npend, upl, ubeg;
  unsigned inv_s, inv_wq;
};

template <int D, int G, int BITS, bool FOLD>
__global__ __launch_bounds__(256, 2) void k_decode_attend(DecodeHot H, Pools P, DecodeLaunch L) {
  constexpr int KK = D / 32;           // MFMA k-steps = quantisation groups per row
  constexpr int LPR = D / 8;           // lanes per value row
  constexpr int R = 64 / LPR;          // value rows per wave load
  constexpr int NV = 16 / R;           // value loads per tile
  constexpr int HB = (G + 3) / 4;      // lane blocks holding real heads
  constexpr int HPL = G < 4 ? G : 4;   // heads per lane
  const int s = blockIdx.x;                       // grid (splits, units of a layer, layers)
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int tok = lane & 15, blk = lane >> 4;
  const int vrow = lane / LPR, sub = lane % LPR;
  const bool active = blk < HB;
  TRACE(0);
  TRACE_XCD();

  __shared__ __align__(16) float pbuf[4][16][G < 4 ? 4 : G];
  __shared__ __align__(16) float pspare[4][16][4];
  // accumulators of the 4 waves; where LDS allows (kParkRows) every value-row group of a wave parks its own share
  // and the readers add them up, which replaces 8 * G cross-lane exchanges per reduction stage
  constexpr bool kParkRows = R * G * D <= 2048;
  constexpr int RP = kParkRows ? R : 1;
  __shared__ __align__(16) float sm_a[4][RP][G][D];
  __shared__ float sm_m[4][G], sm_l[4][G];
  __shared__ float sm_fo[4][G];                        // factor the parked Original-row sums still have to take
  // the waves' sums over packed rows; launches that update the scores put them where the waiting steps' state was
  // (sm_pend: dead by then, a barrier separates the two uses), which keeps two workgroups per compute unit
  __shared__ __align__(16) float sm_q_own[FOLD ? 1 : 4][FOLD ? 1 : G][FOLD ? 4 : D];
  // a block's probabilities, [head][token], rows >= G zero (pitch 80 bytes: the 16 rows a quarter wave reads as
  // 16-byte vectors fall into different bank groups)
  __shared__ __align__(16) _Float16 sm_p[4][16][kVBlock + 8];
  __shared__ _Float16 sm_pdump[4][16][8];
  __shared__ int sm_last;
  __shared__ __align__(16) PendingLds<D, G> sm_pend;   // only touched when FOLD (16-byte alignment: its rows are read as 16-byte vectors)
  static_assert(!FOLD || sizeof(PendingLds<D, G>) >= sizeof(float) * 4 * G * D, "the packed rows' sums must fit the waiting steps' state");
  float (*sm_q)[G][D] = FOLD ? reinterpret_cast<float (*)[G][D]>(&sm_pend) : reinterpret_cast<float (*)[G][D]>(&sm_q_own[0][0][0]);

  // Everything the first tile request depends on is read from the launch arguments in ONE batch of scalar
  // loads (the empty asm pins the values here); left to itself the compiler fetches each where it is first
  // used, six dependent round trips before the first request to HBM.
  // (known counts come with single-layer launches only, so their index is the block index: its address does not
  // wait for units_per_layer, and every launch argument is requested in the same batch)
  const int lk = blockIdx.y < (unsigned)kMaxUnitsKnown ? (int)blockIdx.y : 0;
  int cO = L.cnt_o[lk], cQ = L.cnt_q[lk];
  const int known = H.known, wq = H.wq, splits = H.splits, npend = H.npend;
  const int capO = H.capO, capQ = H.capQ;
  const size_t fin_stride = H.fin_stride;
  const uint16_t* const pok = H.ok;
  const uint16_t* const pov = H.ov;
  float2* const poacc = H.oacc;
  float2* const pqacc = H.qacc;
  const uint16_t* const pq = H.q;
  const int upl = H.upl, ubeg = H.ubeg;
  const unsigned inv_s = H.inv_s, inv_wq = H.inv_wq;
  const float scale2 = L.scale2[blockIdx.z];
  asm volatile("" ::"s"(cO), "s"(cQ), "s"(known), "s"(wq), "s"(splits), "s"(npend), "s"(capO), "s"(capQ),
               "s"(fin_stride), "s"(pok), "s"(pov), "s"(poacc), "s"(pqacc), "s"(pq), "s"(upl), "s"(ubeg), "s"(inv_s),
               "s"(inv_wq), "s"(scale2));
  const int lu = (int)blockIdx.z * upl + (int)blockIdx.y;
  const int gu = ubeg + lu;
  // token counts: from the launch arguments when the host knows them, else from the unit's counters
  if (!known) {
    const volatile int* cnt = reinterpret_cast<const volatile int*>(P.cnt + gu);
    cO = cnt[0]; cQ = cnt[1];
  }

  int ao, bo, aq, bq;
  split_range(cO, cQ, wq, splits, s, SplitRecip{inv_s, inv_wq}, ao, bo, aq, bq);

  const uint16_t* ok_ = pok + (size_t)gu * capO * D;
  const uint16_t* ov_ = pov + (size_t)gu * capO * D;
  float2* oacc_ = poacc + (size_t)gu * capO;
  float2* qacc_ = pqacc + (size_t)gu * capQ;

  // Launches that update the scores at group size 8 work through four rounds of waiting steps per tile and have
  // no registers for a second tile's value rows: those are requested when the tile's turn comes, in front of
  // the score update (which covers their latency), and live in one shared set of registers.
  constexpr bool kLateVO = FOLD && G > 4;
  struct OTile { uint4 kb[KK]; uint4 vr[kLateVO ? 1 : NV]; float2 ac; };
  uint4 vlate[kLateVO ? NV : 1];
  auto load_v = [&](uint4 (&vr)[NV], int row0) {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int rv = min(row0 + R * j + vrow, bo - 1);
      vr[j] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(ov_) + (unsigned)rv * (2 * D) + 16 * sub);
    }
  };
  auto load_o = [&](OTile& t, int row0) {
    const int rk = min(row0 + tok, bo - 1);
    {
      const unsigned off = (unsigned)rk * (2 * D) + 16 * blk;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        t.kb[kk] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(ok_) + off + 64 * kk);
    }
    if constexpr (!kLateVO) load_v(t.vr, row0);
    if constexpr (FOLD) t.ac = oacc_[rk];
  };
  // the first tile is requested before anything else touches memory
  OTile ta, tb;
  if (ao < bo) load_o(ta, ao + 16 * w);
  TRACE(1);

  // this step's query; on a launch that also updates the scores, the waiting steps' state goes to LDS
  uint4 qa[KK];
  load_query<D, G>(pq + (size_t)lu * G * D, lane, qa);
  if constexpr (FOLD) stage_pending<D, G>(P, gu, npend, L.slot, sm_pend, tid, BITS != 8 && cQ > 0, pq + (size_t)lu * G * D);

  float Mreg[HPL], lsum[HPL], acc[G][8];
#pragma unroll
  for (int i = 0; i < HPL; ++i) { Mreg[i] = kNegBig; lsum[i] = 0.f; }
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[h][c] = 0.f;

  // logits x[] of this lane's token -> reference-max check, probabilities, PV with the tile's value rows
  auto softmax_pv = [&](bool live, const float (&x)[HPL], auto&& value_row) {
    bool need = false;
#pragma unroll
    for (int i = 0; i < HPL; ++i) need |= active && (x[i] > Mreg[i] + 8.0f);
    if (__any(need)) {
      float f[HPL];
#pragma unroll
      for (int i = 0; i < HPL; ++i) {
        const float nm = fmaxf(Mreg[i], row_max16(x[i]));
        f[i] = fexp2(Mreg[i] - nm);
        Mreg[i] = nm;
        lsum[i] *= f[i];
      }
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float fh = __builtin_bit_cast(
            float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, f[h % 4]), 16 * (h / 4)));
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[h][c] *= fh;
      }
    }
    float p[HPL];
#pragma unroll
    for (int i = 0; i < HPL; ++i) { p[i] = live ? fexp2(x[i] - Mreg[i]) : 0.f; lsum[i] += p[i]; }
    {
      // every lane stores (inactive blocks into a spare copy of the buffer): no branch around the LDS op
      float* dst = active ? &pbuf[w][tok][4 * blk] : &pspare[w][tok][0];
      if constexpr (HPL == 4) {
        *reinterpret_cast<float4*>(dst) = make_float4(p[0], p[1], p[2], p[3]);
      } else {
#pragma unroll
        for (int i = 0; i < HPL; ++i) dst[i] = p[i];
      }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const float* pp = &pbuf[w][R * j + vrow][0];
      float vf[8];
      value_row(j, vf);                        // 8 channels of value row R*j + vrow as floats
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float ph = pp[h];
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[h][c] = fmaf(ph, vf[c], acc[h][c]);
      }
    }
    __builtin_amdgcn_wave_barrier();
  };

  // deferred score update of the lane's token (FOLD launches only).  The store is predicated: a skipped
  // store only makes a later wait count conservative by one.
  auto store_acc = [&](float2 ac, bool own, float2* acp, int row) {
    if (own && blk == 0) acp[row] = ac;
  };

  // ---------------- Original rows ----------------
  auto compute_o = [&](const OTile& t, int row0) {
    if constexpr (kLateVO) load_v(vlate, row0);
    const f32x4 C = dots_bf16<KK>(qa, t.kb);
    const bool own = (row0 + tok < bo) && active;
    float x[HPL];
#pragma unroll
    for (int i = 0; i < HPL; ++i) x[i] = own ? C[i] * scale2 : kNegBig;
    if constexpr (FOLD) {
      // the token appended by waiting step j sits at row cO - npend + j: older steps did not see it
      const int row = min(row0 + tok, bo - 1);
      const float2 ac = fold_pending<D, G>(sm_pend, npend, row - (cO - npend), t.ac, lane, [&](int, const uint4 (&qop)[KK], float (&xp)[HPL]) {
        const f32x4 Cp = dots_bf16<KK>(qop, t.kb);
#pragma unroll
        for (int i = 0; i < HPL; ++i) xp[i] = Cp[i];
      });
      store_acc(ac, own, oacc_, row);
    }
    softmax_pv(own, x, [&](int j, float (&f)[8]) {
      if constexpr (kLateVO) unpack_bf16x8(vlate[j], f);
      else unpack_bf16x8(t.vr[j], f);
    });
  };
  if (ao < bo) {
    // two tiles in registers: while one is consumed the other is in flight.  Loads past the end of the
    // range are clamped to its last row; every load in the loop is unconditional so that the wait
    // counts the compiler derives are exact and a prefetch is never drained early.
    int row0 = ao + 16 * w;
    for (; row0 + 128 < bo; row0 += 128) {      // this wave still has two more tiles after this one
      load_o(tb, row0 + 64);
      compute_o(ta, row0);
      load_o(ta, row0 + 128);
      compute_o(tb, row0 + 64);
    }
    if (row0 < bo) {                            // one or two tiles left
      load_o(tb, row0 + 64);
      compute_o(ta, row0);
      if (row0 + 64 < bo) compute_o(tb, row0 + 64);
    }
  }

  TRACE(2);
  // ---------------- the token being generated (last split; wave 3 has the fewest tiles) ----------------
  if (s == splits - 1 && w == 3) {
    const uint16_t* kn = L.k_new + (size_t)lu * D;
    const uint16_t* vn = L.v_new + (size_t)lu * D;
    uint4 kb[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kb[kk] = *reinterpret_cast<const uint4*>(kn + 32 * kk + 8 * blk);
    const uint4 vr = *reinterpret_cast<const uint4*>(vn + sub * 8);
    const f32x4 C = dots_bf16<KK>(qa, kb);
    const bool own = (tok == 0) && active;
    float x[HPL];
#pragma unroll
    for (int i = 0; i < HPL; ++i) x[i] = own ? C[i] * scale2 : kNegBig;
    softmax_pv(own, x, [&](int, float (&f)[8]) { unpack_bf16x8(vr, f); });
    uint16_t* dk = P.ok + ((size_t)gu * P.capO + cO) * D;
    uint16_t* dv = P.ov + ((size_t)gu * P.capO + cO) * D;
    if (tok == 0) {
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) *reinterpret_cast<uint4*>(dk + 32 * kk + 8 * blk) = kb[kk];
    }
    if (vrow == 0) *reinterpret_cast<uint4*>(dv + sub * 8) = vr;
    if (lane == 0) {
      P.oacc[(size_t)gu * P.capO + cO] = make_float2(0.f, 0.f);
      P.opos[(size_t)gu * P.capO + cO] = L.position;
      P.qscale[(size_t)L.slot * (P.fin_stride / G) + gu] = scale2;
    }
    // this step's query, for the later launch that adds this step to the scores
    if (tok < G) {
      uint16_t* dq = P.qprev + ((size_t)L.slot * P.fin_stride + (size_t)gu * G + tok) * D + 8 * blk;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) *reinterpret_cast<uint4*>(dq + 32 * kk) = qa[kk];
    }
  }

  TRACE(3);
  // ---------------- the wave's sums over Original rows go to LDS ----------------
  // (where LDS allows, kParkRows, every value-row group parks its own share and the readers add them up)
  if constexpr (kParkRows) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float4* dst = reinterpret_cast<float4*>(&sm_a[w][vrow][h][sub * 8]);
      dst[0] = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
      dst[1] = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
    }
  } else {
#pragma unroll
    for (int stride = LPR; stride < 64; stride <<= 1)
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[h][c] += __shfl_xor(acc[h][c], stride);
    if (vrow == 0) {
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int c = 0; c < 8; ++c) sm_a[w][0][h][sub * 8 + c] = acc[h][c];
    }
  }
#pragma unroll
  for (int i = 0; i < HPL; ++i) lsum[i] = row_sum16(lsum[i]);
  float fo[HPL];                 // rescaling of the reference after the sums above were parked
#pragma unroll
  for (int i = 0; i < HPL; ++i) fo[i] = 1.0f;

  // ---------------- Quantized rows ----------------
  // Blocks of 32 tokens: logits of two 16-token tiles as above (codes -> bf16 MFMA operands), then PV on the
  // matrix cores from the token-minor value blocks (ValueFmt).  Probabilities are at most 1 here (the reference
  // maximum follows every new maximum), so that probability * scale cannot overflow fp16.
  const bool hasq = aq < bq;                 // uniform over the workgroup
  if (__builtin_expect(hasq, 0)) {           // (out of line: most workgroups of a mixed cache hold bf16 rows only)
    using Fmt = PackedFmt<D, HPL, BITS>;
    using VF = ValueFmt<D, BITS>;
    const uint8_t* kc = P.qkc + (size_t)gu * P.capQ * Fmt::CB;
    const uint32_t* km = P.qkm + (size_t)gu * P.capQ * Fmt::NG;
    const uint8_t* vc = P.qvc + (size_t)gu * P.capQv * VF::CB;
    const uint16_t* vm = P.qvm + (size_t)gu * P.capQv * VF::MH;
    // launches that also update the scores (grouped formats) read this step's prepared query from LDS, next to the
    // waiting steps' (PendingLds index ROUNDS); the others keep it in registers
    constexpr bool kQueryInLds = FOLD && BITS != 8;
    typename Fmt::Query pqa;
    if constexpr (!kQueryInLds) Fmt::prep(qa, pqa);
    // rows of the probability buffer that no head fills stay zero
    *reinterpret_cast<uint4*>(&sm_p[w][lane >> 2][8 * (lane & 3)]) = make_uint4(0, 0, 0, 0);
    constexpr int RPG = VF::template rpg<G>(), GPA = VF::template gpa<G>(), NA = VF::template na<G>();
    // row tok of A operand j: head tok % RPG, group j * GPA + tok / RPG (rows beyond the groups repeat the last)
    const int arow_head = tok % RPG;
    int gs[VF::NSC];
#pragma unroll
    for (int j = 0; j < VF::NSC; ++j) gs[j] = min(j * GPA + tok / RPG, VF::NG - 1);
    f32x4 pacc[VF::NACC], sacc[NA], zacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int a = 0; a < VF::NACC; ++a) pacc[a] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < NA; ++j) sacc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint4 ones = make_uint4(kOnesF16, kOnesF16, kOnesF16, kOnesF16);
    constexpr bool kLateV = FOLD && BITS != 8;
    struct QBlk { typename Fmt::Keys k[2]; typename VF::Blk v; float2 ac[2]; };
    const int blast = (bq - 1) / kVBlock;      // last block of the range (loads are clamped to it)
    auto load_q = [&](QBlk& t, int b32) {
      b32 = min(b32, blast);
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        const int rk = min(kVBlock * b32 + 16 * tl + tok, bq - 1);
        Fmt::load_keys(kc, km, rk, blk, t.k[tl]);
        if constexpr (FOLD) t.ac[tl] = qacc_[rk];
      }
      // launches that also update the scores spend several times longer on a block's logits (grouped formats):
      // there the value block is requested at the start of the block's work instead of one block ahead, which
      // saves a buffer's worth of registers
      if constexpr (!kLateV) VF::load(vc, vm, b32, tok, blk, gs, NA, t.v);
    };
    auto compute_q = [&](const QBlk& t, int b32) {
      typename VF::Blk vnow;
      if constexpr (kLateV) VF::load(vc, vm, b32, tok, blk, gs, NA, vnow);
      const typename VF::Blk& tv = kLateV ? vnow : t.v;
      float x[2][HPL];
      bool own[2];
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        const int row = kVBlock * b32 + 16 * tl + tok;
        own[tl] = (row < bq) && active;
        if constexpr (kQueryInLds)
          Fmt::dots_pending(sm_pend.qp[PendingShape<G>::ROUNDS], sm_pend.qs[PendingShape<G>::ROUNDS], t.k[tl], tok, blk, x[tl]);
        else
          Fmt::dots(pqa, t.k[tl], x[tl]);
#pragma unroll
        for (int i = 0; i < HPL; ++i) x[tl][i] = own[tl] ? x[tl][i] * scale2 : kNegBig;
        if constexpr (FOLD) {
          const float2 ac = fold_pending<D, G>(sm_pend, npend, 0, t.ac[tl], lane, [&](int r, const uint4 (&qop)[KK], float (&xp)[HPL]) {
            if constexpr (BITS == 8) {
              typename Fmt::Query pq_;
              Fmt::prep(qop, pq_);
              Fmt::dots(pq_, t.k[tl], xp);
            } else {
              Fmt::dots_pending(sm_pend.qp[r], sm_pend.qs[r], t.k[tl], tok, blk, xp);
            }
          });
          store_acc(ac, own[tl], qacc_, min(row, bq - 1));
        }
      }
      bool need = false;
#pragma unroll
      for (int i = 0; i < HPL; ++i) need |= active && (fmaxf(x[0][i], x[1][i]) > Mreg[i]);
      if (__any(need)) {
#pragma unroll
        for (int i = 0; i < HPL; ++i) {
          const float nm = fmaxf(Mreg[i], row_max16(fmaxf(x[0][i], x[1][i])));
          const float f = fexp2(Mreg[i] - nm);      // the same in the 16 lanes of a block; 1 in blocks without heads
          Mreg[i] = nm;
          lsum[i] *= f;
          fo[i] *= f;
          zacc[i] *= f;                             // rows of the correction MFMA are the heads, as in this layout
          // rows of the PV accumulators: head (4 blk + i) % RPG, whose factor lives in lane block that head / 4
          float fr;
          if constexpr (RPG == 16) fr = f;
          else if constexpr (RPG == 4) fr = lane_value(f, 0);
          else fr = (blk & 1) ? lane_value(f, 16) : lane_value(f, 0);
#pragma unroll
          for (int a = 0; a < VF::NACC; ++a) pacc[a][i] *= fr;
#pragma unroll
          for (int j = 0; j < NA; ++j) sacc[j][i] *= fr;
        }
      }
      // probabilities as fp16, [head][token] (blocks without heads write a dump: no branch round the LDS op)
#pragma unroll
      for (int tl = 0; tl < 2; ++tl)
#pragma unroll
        for (int i = 0; i < HPL; ++i) {
          const float p = own[tl] ? fexp2(x[tl][i] - Mreg[i]) : 0.f;
          _Float16* dst = active ? &sm_p[w][4 * blk + i][16 * tl + tok] : &sm_pdump[w][tok][4 * tl + i];
          *dst = (_Float16)p;
        }
      __builtin_amdgcn_wave_barrier();
      const uint4 pz = *reinterpret_cast<const uint4*>(&sm_p[w][tok][8 * blk]);        // row = head lane%16, tokens 8 (lane/16) ..+7
      uint4 pg = pz;
      if constexpr (RPG != 16) pg = *reinterpret_cast<const uint4*>(&sm_p[w][arow_head][8 * blk]);   // row = head of a group's row
      __builtin_amdgcn_wave_barrier();
      zacc = mfma16h(pz, tv.z, zacc);
#pragma unroll
      for (int j = 0; j < NA; ++j) {
        const uint4 aj = mul_f16x8(pg, tv.sc[j]);
        if constexpr (VF::kBiased) sacc[j] = mfma16h(aj, ones, sacc[j]);
#pragma unroll
        for (int a = j * GPA * VF::APG; a < (j + 1) * GPA * VF::APG && a < VF::NACC; ++a)
          pacc[a] = mfma16h(aj, VF::operand(tv, a, tok), pacc[a]);
      }
    };
    QBlk qa_, qb_;
    int b32 = aq / kVBlock + w;                // aq is a multiple of the block size
    load_q(qa_, b32);
    for (; b32 + 8 <= blast; b32 += 8) {
      load_q(qb_, b32 + 4);
      compute_q(qa_, b32);
      load_q(qa_, b32 + 8);
      compute_q(qb_, b32 + 4);
    }
    if (b32 <= blast) {
      load_q(qb_, b32 + 4);
      compute_q(qa_, b32);
      if (b32 + 4 <= blast) compute_q(qb_, b32 + 4);
    }
    if constexpr (FOLD) __syncthreads();      // every wave is done with the waiting steps' state (hasq is uniform)
    // accumulators -> channel sums: take the code offset out (1024 * sum of the A operand), undo the code's
    // position in its byte, add the zero points' share (column g of the correction MFMA, whose rows are the heads)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float lq = __shfl(zacc[i], (lane & 48) | VF::ZCOLS);
      if (i < HPL) lsum[i] += lq;
#pragma unroll
      for (int a = 0; a < VF::NACC; ++a) {
        const int g = VF::group_of(a), j = g / GPA;
        const int r0 = RPG == 16 ? 0 : (g % GPA) * RPG;          // first operand row of this group
        const int head = 4 * blk + i - r0;
        const bool useful = head >= 0 && head < G;
        float v = pacc[a][i];
        if constexpr (VF::kBiased) v = fmaf(-1024.0f, sacc[j][i], v);
        float zg = 0.f;
        if constexpr (VF::ZCOLS > 0) zg = __shfl(zacc[i], (16 * max(blk - r0 / 4, 0)) | g);
        v = fmaf(v, VF::unscale(a, tok), zg);
        if (useful) sm_q[w][head][VF::channel(a, tok)] = v;
      }
    }
  }

  TRACE(4);
  // ---------------- across the 4 waves ----------------
  if (tok == 0 && active) {
#pragma unroll
    for (int i = 0; i < HPL; ++i) { sm_m[w][4 * blk + i] = Mreg[i]; sm_l[w][4 * blk + i] = lsum[i]; sm_fo[w][4 * blk + i] = fo[i]; }
  }
  __syncthreads();

  // ---------------- this split's partial ----------------
  float* part = P.part + ((size_t)(gu - L.part_unit0) * P.max_splits + s) * G * (D + 2);
  for (int idx = tid; idx < G * D / 2; idx += 256) {
    const int h = idx / (D / 2), c = 2 * (idx % (D / 2));
    float M = sm_m[0][h];
#pragma unroll
    for (int i = 1; i < 4; ++i) M = fmaxf(M, sm_m[i][h]);
    float a0 = 0.f, a1 = 0.f, l = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float cw_ = fexp2(sm_m[i][h] - M);
      // the wave's value-row groups, added pairwise in the order a butterfly over the lanes would take
      float2 t[RP];
#pragma unroll
      for (int v = 0; v < RP; ++v) t[v] = *reinterpret_cast<const float2*>(&sm_a[i][v][h][c]);
#pragma unroll
      for (int st = 1; st < RP; st <<= 1)
#pragma unroll
        for (int v = 0; v < RP; v += 2 * st) { t[v].x += t[v + st].x; t[v].y += t[v + st].y; }
      if (hasq) {
        const float2 tq = *reinterpret_cast<const float2*>(&sm_q[i][h][c]);
        const float f = sm_fo[i][h];
        t[0].x = fmaf(t[0].x, f, tq.x);
        t[0].y = fmaf(t[0].y, f, tq.y);
      }
      a0 = fmaf(t[0].x, cw_, a0);
      a1 = fmaf(t[0].y, cw_, a1);
      l = fmaf(sm_l[i][h], cw_, l);
    }
    st_dev2(part + h * (D + 2) + c, a0, a1);
    if (c == 0) st_dev2(part + h * (D + 2) + D, M, l);
  }

  TRACE(5);
  // ---------------- the unit's last workgroup merges ----------------
  // Every lane waits until its own stores are acknowledged, the barrier collects the workgroup, then one
  // lane takes a ticket.  The workgroup that draws the last ticket of the unit sees all partials.
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (tid == 0) {
    int* const ticket = P.ticket + (gu - L.part_unit0);
    const int old = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = old == splits - 1;
    if (last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
    sm_last = last;
  }
  __syncthreads();
  if (sm_last) combine_splits<D, G>(P, L, lu, gu, tid);
  TRACE(6);
}

// The deferred score update on its own (before a tailor or an export): the same fold as in
// k_decode_attend, over all rows of the unit.
// grid (workgroups per unit, units); a wave takes every (4 * gridDim.x)-th tile of 16 rows.
template <int D, int G, int BITS>
__global__ __launch_bounds__(256) void k_flush_scores(Pools P, int unit_begin, int n_pending, int slot) {
  constexpr int KK = D / 32;
  constexpr int HPL = G < 4 ? G : 4;
  __shared__ __align__(16) PendingLds<D, G> sm_pend;
  const int gu = unit_begin + blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int tok = lane & 15, blk = lane >> 4;
  const int2 cnt = P.cnt[gu];
  stage_pending<D, G>(P, gu, n_pending, slot, sm_pend, threadIdx.x, BITS != 8 && cnt.y > 0);
  const int wave = blockIdx.x * 4 + w, step = gridDim.x * 64;
  {
    const uint16_t* ok_ = P.ok + (size_t)gu * P.capO * D;
    float2* acc = P.oacc + (size_t)gu * P.capO;
    for (int row0 = 16 * wave; row0 < cnt.x; row0 += step) {
      const int rk = min(row0 + tok, cnt.x - 1);
      uint4 kb[KK];
      const unsigned off = (unsigned)rk * (2 * D) + 16 * blk;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        kb[kk] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(ok_) + off + 64 * kk);
      // the token appended by waiting step j sits at row cnt.x - n_pending + j
      const float2 ac = fold_pending<D, G>(sm_pend, n_pending, rk - (cnt.x - n_pending), acc[rk], lane,
                                           [&](int, const uint4 (&qop)[KK], float (&xp)[HPL]) {
        const f32x4 Cp = dots_bf16<KK>(qop, kb);
#pragma unroll
        for (int i = 0; i < HPL; ++i) xp[i] = Cp[i];
      });
      if (row0 + tok < cnt.x && blk == 0) acc[rk] = ac;
    }
  }
  if (cnt.y > 0) {
    using Fmt = PackedFmt<D, HPL, BITS>;
    const uint8_t* kc = P.qkc + (size_t)gu * P.capQ * Fmt::CB;
    const uint32_t* km = P.qkm + (size_t)gu * P.capQ * Fmt::NG;
    float2* acc = P.qacc + (size_t)gu * P.capQ;
    for (int row0 = 16 * wave; row0 < cnt.y; row0 += step) {
      const int rk = min(row0 + tok, cnt.y - 1);
      typename Fmt::Keys k;
      Fmt::load_keys(kc, km, rk, blk, k);
      const float2 ac = fold_pending<D, G>(sm_pend, n_pending, 0, acc[rk], lane, [&](int r, const uint4 (&qop)[KK], float (&xp)[HPL]) {
        if constexpr (BITS == 8) {
          typename Fmt::Query pq_;
          Fmt::prep(qop, pq_);
          Fmt::dots(pq_, k, xp);
        } else {
          Fmt::dots_pending(sm_pend.qp[r], sm_pend.qs[r], k, tok, blk, xp);
        }
      });
      if (row0 + tok < cnt.y && blk == 0) acc[rk] = ac;
    }
  }
}

template <int D, int G, int BITS>
static hipError_t launch_decode_t(const Pools& P, const DecodeLaunch& a, hipStream_t s, hipEvent_t ev0,
                                  hipEvent_t ev1) {
  dim3 grid(a.splits, a.units_per_layer, a.n_units / a.units_per_layer);
  if (ev0) (void)hipEventRecord(ev0, s);
#ifdef ARKV_PHASE_TRACE
  hipLaunchKernelGGL(k_trace_mark, dim3(1), dim3(64), 0, s, 0);
#endif
  DecodeHot h;
  h.ok = P.ok; h.ov = P.ov; h.oacc = P.oacc; h.qacc = P.qacc; h.q = a.q;
  h.fin_stride = P.fin_stride;
  h.capO = P.capO; h.capQ = P.capQ; h.splits = a.splits; h.wq = a.wq; h.known = a.cnt_known; h.npend = a.n_pending;
  h.upl = a.units_per_layer; h.ubeg = a.unit_begin; h.inv_s = a.inv_splits; h.inv_wq = a.inv_wq;
  if (a.fold) hipLaunchKernelGGL((k_decode_attend<D, G, BITS, true>), grid, dim3(256), 0, s, h, P, a);
  else hipLaunchKernelGGL((k_decode_attend<D, G, BITS, false>), grid, dim3(256), 0, s, h, P, a);
#ifdef ARKV_PHASE_TRACE
  hipLaunchKernelGGL(k_trace_mark, dim3(1), dim3(64), 0, s, 1);
#endif
  if (ev1) (void)hipEventRecord(ev1, s);
  return hipGetLastError();
}

template <int D, int G>
static hipError_t launch_decode_b(const Pools& P, const DecodeLaunch& a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  if (P.bits == 8) return launch_decode_t<D, G, 8>(P, a, s, e0, e1);
  return P.bits == 4 ? launch_decode_t<D, G, 4>(P, a, s, e0, e1) : launch_decode_t<D, G, 2>(P, a, s, e0, e1);
}

template <int D>
static hipError_t launch_decode_g(const Pools& P, const DecodeLaunch& a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  switch (P.G) {
    case 1: return launch_decode_b<D, 1>(P, a, s, e0, e1);
    case 2: return launch_decode_b<D, 2>(P, a, s, e0, e1);
    case 4: return launch_decode_b<D, 4>(P, a, s, e0, e1);
    case 8: return launch_decode_b<D, 8>(P, a, s, e0, e1);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_decode(const Pools& P, const DecodeLaunch& a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  if (P.D == 128) return launch_decode_g<128>(P, a, s, e0, e1);
  if (P.D == 64) return launch_decode_g<64>(P, a, s, e0, e1);
  return hipErrorInvalidValue;
}

// ---- split-K scratch for callers that cannot allocate ---------------------------------------------
// One file-scope array per GPU: the units' tickets first (zero between launches: the workgroup that draws a
// unit's last ticket clears it), the splits' partials behind them.  The array's name is only a handle in host
// code; its device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static unsigned char* g_scratch_ptr[kMaxDevices] = {};

__global__ void k_clear_words(unsigned* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

hipError_t static_scratch_setup() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (g_scratch_ptr[dev]) return hipSuccess;
  unsigned char* ptr = nullptr;
  e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!ptr) return hipErrorInvalidSymbol;
  hipLaunchKernelGGL(k_clear_words, dim3((kStaticUnits + 255) / 256), dim3(256), 0, nullptr,
                     reinterpret_cast<unsigned*>(ptr), kStaticUnits);
  e = hipGetLastError();
  if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
  if (e != hipSuccess) return e;
  g_scratch_ptr[dev] = ptr;
  return hipSuccess;
}

hipError_t static_scratch_get(float** part, int** ticket, size_t* part_floats) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices || !g_scratch_ptr[dev]) return hipErrorNotInitialized;
  unsigned char* ptr = g_scratch_ptr[dev];
  *ticket = reinterpret_cast<int*>(ptr);
  *part = reinterpret_cast<float*>(ptr + (size_t)kStaticUnits * sizeof(int));
  *part_floats = (kStaticScratchBytes - (size_t)kStaticUnits * sizeof(int)) / sizeof(float);
  return hipSuccess;
}

// which: 0 = the decode kernel's phase marks, 1 = its merge marks; n_wg rows of 8 words each
hipError_t phase_trace_decode(int which, unsigned long long* host, int n_wg, bool* built) {
#ifdef ARKV_PHASE_TRACE
  *built = true;
  if (n_wg < 0 || n_wg > 8192) return hipErrorInvalidValue;
  const size_t bytes = (size_t)n_wg * 8 * sizeof(unsigned long long);
  return which == 0 ? hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), bytes)
                    : hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace_m), bytes);
#else
  (void)which; (void)host; (void)n_wg;
  *built = false;
  return hipSuccess;
#endif
}

template <int D, int G>
static hipError_t launch_flush_b(const Pools& P, dim3 grid, int unit_begin, int n_pending, int slot, hipStream_t s) {
  if (P.bits == 8) hipLaunchKernelGGL((k_flush_scores<D, G, 8>), grid, dim3(256), 0, s, P, unit_begin, n_pending, slot);
  else if (P.bits == 4) hipLaunchKernelGGL((k_flush_scores<D, G, 4>), grid, dim3(256), 0, s, P, unit_begin, n_pending, slot);
  else hipLaunchKernelGGL((k_flush_scores<D, G, 2>), grid, dim3(256), 0, s, P, unit_begin, n_pending, slot);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_flush_g(const Pools& P, dim3 grid, int unit_begin, int n_pending, int slot, hipStream_t s) {
  switch (P.G) {
    case 1: return launch_flush_b<D, 1>(P, grid, unit_begin, n_pending, slot, s);
    case 2: return launch_flush_b<D, 2>(P, grid, unit_begin, n_pending, slot, s);
    case 4: return launch_flush_b<D, 4>(P, grid, unit_begin, n_pending, slot, s);
    case 8: return launch_flush_b<D, 8>(P, grid, unit_begin, n_pending, slot, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_flush_scores(const Pools& P, int unit_begin, int n_units, int n_pending, int slot, hipStream_t s) {
  const int cap = P.capO > P.capQ ? P.capO : P.capQ;
  int bx = (cap + 63) / 64;               // one tile per wave at most
  if (bx > 32) bx = 32;
  const dim3 grid(bx, n_units);
  if (P.D == 128) return launch_flush_g<128>(P, grid, unit_begin, n_pending, slot, s);
  if (P.D == 64) return launch_flush_g<64>(P, grid, unit_begin, n_pending, slot, s);
  return hipErrorInvalidValue;
}

}  // namespace arkv

extern "C" int arkv_debug_split_range(int32_t n_original, int32_t n_quantized, int32_t packed_weight, int32_t n_splits,
                                      int32_t split, int32_t* range) {
  if (!range || n_original < 0 || n_quantized < 0 || n_splits < 1 || n_splits > arkv::kMaxSplits || split < 0 ||
      split >= n_splits || packed_weight < 1 || packed_weight > 16 ||
      (16ull * (uint64_t)n_original + (uint64_t)packed_weight * (uint64_t)n_quantized + 512ull) * (uint64_t)n_splits > 0xFFFFFFFFull)
    return ARKV_EINVAL;
  int ao, bo, aq, bq;
  arkv::split_range(n_original, n_quantized, packed_weight, n_splits, split, arkv::split_recip(n_splits, packed_weight), ao, bo,
                    aq, bq);
  range[0] = ao; range[1] = bo; range[2] = aq; range[3] = bq;
  return ARKV_OK;
}

