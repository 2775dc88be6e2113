// Decode step kernels (Alg. 1 "Decoding Phase" + "Reconstruction Before Attention", fused):
//   k_decode_attend : append + split-K attention of one query per head over the bf16 pool and the
//                     packed low-bit pool (dequantisation inside the QK and PV loops) + the score
//                     update of the PREVIOUS step (its probabilities need that step's final
//                     softmax denominator, which only exists after the split-K combine)
//   k_decode_combine: merges the split-K partials, writes the output and the step's (max, 1/sum)
//   k_flush_scores  : adds the pending probabilities to (s1, s2) when something needs them now
//                     (tailor, export)
#include <hip/hip_fp16.h>

#include "arkv_dev.h"

namespace arkv {

constexpr float kNegBig = -1.0e30f;

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL,
                                                               0xf, 0xf, true));
}

// Sum over the LPR consecutive lanes that share a row (LPR = 8 or 16, aligned); every lane gets the sum.
template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_mov<0xB1>(x);                 // quad_perm [1,0,3,2]
  x += dpp_mov<0x4E>(x);                 // quad_perm [2,3,0,1]
  x += dpp_mov<0x141>(x);                // row_half_mirror: lane i <- 7-i
  if (LPR >= 16) x += dpp_mov<0x140>(x); // row_mirror: lane i <- 15-i
  return x;
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

// 8 consecutive channels of a packed row -> fp32 values code*scale + zero.
template <int BITS>
__device__ __forceinline__ void dequant8(uint32_t codes, uint32_t meta, float (&f)[8]) {
  const float sc = half_bits_to_float(meta), z = half_bits_to_float(meta >> 16);
  constexpr uint32_t mask = (1u << BITS) - 1u;
#pragma unroll
  for (int c = 0; c < 8; ++c) f[c] = fmaf((float)((codes >> (BITS * c)) & mask), sc, z);
}

__device__ __forceinline__ uint16_t float_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Rows [ao,bo) of the O pool and [aq,bq) of the Q pool that split s of S owns.  Rows are weighted
// by their bytes (bf16 row = 16 units, packed row = wq units) so that splits stream equal bytes.
__host__ __device__ inline void split_range(int cO, int cQ, int wq, int S, int s, int& ao, int& bo,
                                            int& aq, int& bq) {
  const long long tot = 16LL * cO + (long long)wq * cQ;
  const long long v0 = tot * s / S, v1 = tot * (s + 1) / S;
  auto mapO = [&](long long v) { long long r = (v + 15) / 16; return (int)(r < cO ? r : cO); };
  auto mapQ = [&](long long v) {
    long long w = v - 16LL * cO;
    if (w <= 0) return 0;
    long long r = (w + wq - 1) / wq;
    return (int)(r < cQ ? r : cQ);
  };
  ao = mapO(v0); bo = mapO(v1); aq = mapQ(v0); bq = mapQ(v1);
}

template <int G>
struct Softmax {
  float m[G], l[G], a[G][8];
};

// One tile of UNR rows per lane group: logits, online softmax update, PV accumulation.
template <int LPR, int G, int UNR>
__device__ __forceinline__ void consume(Softmax<G>& st, const float (&qf)[G][8], const float (&kf)[UNR][8],
                                        const float (&vf)[UNR][8], const bool (&ok)[UNR], float scale2,
                                        float (&lg)[UNR][G]) {
#pragma unroll
  for (int u = 0; u < UNR; ++u) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float d = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) d = fmaf(qf[h][c], kf[u][c], d);
      d = group_sum<LPR>(d);
      lg[u][h] = ok[u] ? d * scale2 : kNegBig;
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float mt = lg[0][h];
#pragma unroll
    for (int u = 1; u < UNR; ++u) mt = fmaxf(mt, lg[u][h]);
    const float mn = fmaxf(st.m[h], mt);
    const float corr = exp2f(st.m[h] - mn);
    st.m[h] = mn;
    st.l[h] *= corr;
#pragma unroll
    for (int c = 0; c < 8; ++c) st.a[h][c] *= corr;
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const float p = ok[u] ? exp2f(lg[u][h] - mn) : 0.f;
      st.l[h] += p;
#pragma unroll
      for (int c = 0; c < 8; ++c) st.a[h][c] = fmaf(p, vf[u][c], st.a[h][c]);
    }
  }
}

template <int G>
__device__ __forceinline__ void merge(Softmax<G>& x, const Softmax<G>& y) {
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const float M = fmaxf(x.m[h], y.m[h]);
    const float cx = exp2f(x.m[h] - M), cy = exp2f(y.m[h] - M);
    x.m[h] = M;
    x.l[h] = x.l[h] * cx + y.l[h] * cy;
#pragma unroll
    for (int c = 0; c < 8; ++c) x.a[h][c] = x.a[h][c] * cx + y.a[h][c] * cy;
  }
}

template <int G>
__device__ __forceinline__ void store_logits(float* dst, const float (&lg)[G]) {
  if constexpr (G == 4) {
    *reinterpret_cast<float4*>(dst) = make_float4(lg[0], lg[1], lg[2], lg[3]);
  } else {
#pragma unroll
    for (int h = 0; h < G; ++h) dst[h] = lg[h];
  }
}

// (s1, s2) += sum_h p_h, sum_h p_h^2 with p_h = 2^(lg_h - m_h) / Z_h, slots [a, b), one thread per slot.
template <int G>
__device__ __forceinline__ void apply_pending(float2* acc, const float* lg, int a, int b,
                                              const float (&pm)[G], const float (&pinv)[G], int tid,
                                              int nthreads) {
  for (int i = a + tid; i < b; i += nthreads) {
    float v[G];
    if constexpr (G == 4) {
      const float4 t = *reinterpret_cast<const float4*>(lg + (size_t)i * G);
      v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
      for (int h = 0; h < G; ++h) v[h] = lg[(size_t)i * G + h];
    }
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float p = exp2f(v[h] - pm[h]) * pinv[h];
      s1 += p;
      s2 = fmaf(p, p, s2);
    }
    float2 t = acc[i];
    t.x += s1; t.y += s2;
    acc[i] = t;
  }
}

template <int D, int G, int BITS>
__global__ __launch_bounds__(256) void k_decode_attend(Pools P, DecodeLaunch L) {
  constexpr int LPR = D / 8;        // lanes per row
  constexpr int R = 64 / LPR;       // rows per wave per load
  constexpr int UNR = 4;
  constexpr int TILE = 4 * R * UNR; // rows per workgroup iteration
  constexpr int CB = D * BITS / 8;  // code bytes per row
  constexpr int NG = D / kGroup;
  const int s = blockIdx.x, lu = blockIdx.y;
  const int gu = L.unit_begin + lu;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int rg = lane / LPR, sub = lane % LPR;
  const float scale2 = L.scale2[lu / L.units_per_layer];

  const int2 cnt = P.cnt[gu];
  const int cO = cnt.x, cQ = cnt.y;
  int ao, bo, aq, bq;
  split_range(cO, cQ, BITS == 4 ? 5 : 3, L.splits, s, ao, bo, aq, bq);

  const uint16_t* ok_ = P.ok + (size_t)gu * P.capO * D;
  const uint16_t* ov_ = P.ov + (size_t)gu * P.capO * D;
  float* olg = P.olg + (size_t)gu * P.capO * G;
  float* qlg = P.qlg + (size_t)gu * P.capQ * G;
  float2* oacc = P.oacc + (size_t)gu * P.capO;
  float2* qacc = P.qacc + (size_t)gu * P.capQ;

  // ---- phase 1: fold the previous step's probabilities into (s1, s2) for the rows this split owns
  if (L.has_pending) {
    float pm[G], pinv[G];
    const float2* f = P.fin + (size_t)L.parity * P.fin_stride + (size_t)gu * G;
#pragma unroll
    for (int h = 0; h < G; ++h) { pm[h] = f[h].x; pinv[h] = f[h].y; }
    apply_pending<G>(oacc, olg, ao, bo, pm, pinv, tid, 256);
    apply_pending<G>(qacc, qlg, aq, bq, pm, pinv, tid, 256);
    __syncthreads();   // the main loop overwrites these logits from other threads
  }

  // ---- query of this unit's G heads: the 8 channels this lane owns
  float qf[G][8];
  {
    const uint16_t* q = L.q + ((size_t)lu * G) * D + sub * 8;
#pragma unroll
    for (int h = 0; h < G; ++h) unpack_bf16x8(*reinterpret_cast<const uint4*>(q + (size_t)h * D), qf[h]);
  }
  Softmax<G> st;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    st.m[h] = kNegBig; st.l[h] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) st.a[h][c] = 0.f;
  }

  // ---- Original rows
  for (int r0 = ao; r0 < bo; r0 += TILE) {
    uint4 kr[UNR], vr[UNR];
    bool ok[UNR];
    int row[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      row[u] = r0 + (u * 4 + w) * R + rg;
      ok[u] = row[u] < bo;
      const int rr = ok[u] ? row[u] : bo - 1;
      kr[u] = *reinterpret_cast<const uint4*>(ok_ + (size_t)rr * D + sub * 8);
      vr[u] = *reinterpret_cast<const uint4*>(ov_ + (size_t)rr * D + sub * 8);
    }
    float kf[UNR][8], vf[UNR][8], lg[UNR][G];
#pragma unroll
    for (int u = 0; u < UNR; ++u) { unpack_bf16x8(kr[u], kf[u]); unpack_bf16x8(vr[u], vf[u]); }
    consume<LPR, G, UNR>(st, qf, kf, vf, ok, scale2, lg);
    if (sub == 0) {
#pragma unroll
      for (int u = 0; u < UNR; ++u)
        if (ok[u]) store_logits<G>(olg + (size_t)row[u] * G, lg[u]);
    }
  }

  // ---- Quantized rows: dequantise in registers
  {
    const uint8_t* kc = P.qkc + (size_t)gu * P.capQ * CB;
    const uint8_t* vc = P.qvc + (size_t)gu * P.capQ * CB;
    const uint32_t* km = P.qkm + (size_t)gu * P.capQ * NG;
    const uint32_t* vm = P.qvm + (size_t)gu * P.capQ * NG;
    for (int r0 = aq; r0 < bq; r0 += TILE) {
      uint32_t kcr[UNR], vcr[UNR], kmr[UNR], vmr[UNR];
      bool ok[UNR];
      int row[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        row[u] = r0 + (u * 4 + w) * R + rg;
        ok[u] = row[u] < bq;
        const int rr = ok[u] ? row[u] : bq - 1;
        if (BITS == 4) {
          kcr[u] = *reinterpret_cast<const uint32_t*>(kc + (size_t)rr * CB + sub * 4);
          vcr[u] = *reinterpret_cast<const uint32_t*>(vc + (size_t)rr * CB + sub * 4);
        } else {
          kcr[u] = *reinterpret_cast<const uint16_t*>(kc + (size_t)rr * CB + sub * 2);
          vcr[u] = *reinterpret_cast<const uint16_t*>(vc + (size_t)rr * CB + sub * 2);
        }
        kmr[u] = km[(size_t)rr * NG + sub / 4];
        vmr[u] = vm[(size_t)rr * NG + sub / 4];
      }
      float kf[UNR][8], vf[UNR][8], lg[UNR][G];
#pragma unroll
      for (int u = 0; u < UNR; ++u) { dequant8<BITS>(kcr[u], kmr[u], kf[u]); dequant8<BITS>(vcr[u], vmr[u], vf[u]); }
      consume<LPR, G, UNR>(st, qf, kf, vf, ok, scale2, lg);
      if (sub == 0) {
#pragma unroll
        for (int u = 0; u < UNR; ++u)
          if (ok[u]) store_logits<G>(qlg + (size_t)row[u] * G, lg[u]);
      }
    }
  }

  // ---- the token being generated: the last split appends it to the O pool and attends to it
  if (s == L.splits - 1) {
    const uint16_t* kn = L.k_new + (size_t)lu * D + sub * 8;
    const uint16_t* vn = L.v_new + (size_t)lu * D + sub * 8;
    const uint4 kr = *reinterpret_cast<const uint4*>(kn);
    const uint4 vr = *reinterpret_cast<const uint4*>(vn);
    float kf[1][8], vf[1][8], lg[1][G];
    bool ok[1] = {w == 0 && rg == 0};
    unpack_bf16x8(kr, kf[0]); unpack_bf16x8(vr, vf[0]);
    consume<LPR, G, 1>(st, qf, kf, vf, ok, scale2, lg);
    if (ok[0]) {
      uint16_t* dk = P.ok + ((size_t)gu * P.capO + cO) * D + sub * 8;
      uint16_t* dv = P.ov + ((size_t)gu * P.capO + cO) * D + sub * 8;
      *reinterpret_cast<uint4*>(dk) = kr;
      *reinterpret_cast<uint4*>(dv) = vr;
      if (sub == 0) {
        store_logits<G>(olg + (size_t)cO * G, lg[0]);
        oacc[cO] = make_float2(0.f, 0.f);
        P.opos[(size_t)gu * P.capO + cO] = L.position;
      }
    }
  }

  // ---- reduce the row groups of a wave, then the 4 waves, and write this split's partial
#pragma unroll
  for (int stride = LPR; stride < 64; stride <<= 1) {
    Softmax<G> o;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      o.m[h] = __shfl_xor(st.m[h], stride);
      o.l[h] = __shfl_xor(st.l[h], stride);
#pragma unroll
      for (int c = 0; c < 8; ++c) o.a[h][c] = __shfl_xor(st.a[h][c], stride);
    }
    merge<G>(st, o);
  }
  __shared__ float sm_a[4][G][D];
  __shared__ float sm_m[4][G], sm_l[4][G];
  if (rg == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
      for (int c = 0; c < 8; ++c) sm_a[w][h][sub * 8 + c] = st.a[h][c];
      if (sub == 0) { sm_m[w][h] = st.m[h]; sm_l[w][h] = st.l[h]; }
    }
  }
  __syncthreads();
  float* part = P.part + ((size_t)gu * kMaxSplits + s) * G * (D + 2);
  for (int idx = tid; idx < G * D; idx += 256) {
    const int h = idx / D, c = idx % D;
    float M = sm_m[0][h];
#pragma unroll
    for (int i = 1; i < 4; ++i) M = fmaxf(M, sm_m[i][h]);
    float a = 0.f, l = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float cw = exp2f(sm_m[i][h] - M);
      a = fmaf(sm_a[i][h][c], cw, a);
      l = fmaf(sm_l[i][h], cw, l);
    }
    part[h * (D + 2) + c] = a;
    if (c == 0) { part[h * (D + 2) + D] = M; part[h * (D + 2) + D + 1] = l; }
  }
}

template <int D, int G>
__global__ __launch_bounds__(256) void k_decode_combine(Pools P, DecodeLaunch L) {
  const int lu = blockIdx.x, gu = L.unit_begin + lu, tid = threadIdx.x;
  const float* part = P.part + (size_t)gu * kMaxSplits * G * (D + 2);
  const int S = L.splits;
  for (int idx = tid; idx < G * D; idx += 256) {
    const int h = idx / D, c = idx % D;
    const float* ph = part + h * (D + 2);
    float M = kNegBig;
    for (int s = 0; s < S; ++s) M = fmaxf(M, ph[(size_t)s * G * (D + 2) + D]);
    float a = 0.f, l = 0.f;
    for (int s = 0; s < S; ++s) {
      const float* p = ph + (size_t)s * G * (D + 2);
      const float cw = exp2f(p[D] - M);
      a = fmaf(p[c], cw, a);
      l = fmaf(p[D + 1], cw, l);
    }
    const float inv = 1.0f / l;
    const float o = a * inv;
    P.outf[((size_t)gu * G + h) * D + c] = o;
    L.out[((size_t)lu * G + h) * D + c] = float_to_bf16_rne(o);
    if (c == 0) P.fin[(size_t)(L.parity ^ 1) * P.fin_stride + (size_t)gu * G + h] = make_float2(M, inv);
  }
  if (tid == 0) P.cnt[gu].x += 1;
}

template <int G>
__global__ __launch_bounds__(256) void k_flush_scores(Pools P, int unit_begin, int parity) {
  const int gu = unit_begin + blockIdx.y;
  const int2 cnt = P.cnt[gu];
  float pm[G], pinv[G];
  const float2* f = P.fin + (size_t)parity * P.fin_stride + (size_t)gu * G;
#pragma unroll
  for (int h = 0; h < G; ++h) { pm[h] = f[h].x; pinv[h] = f[h].y; }
  const int tid = blockIdx.x * 256 + threadIdx.x, nt = gridDim.x * 256;
  apply_pending<G>(P.oacc + (size_t)gu * P.capO, P.olg + (size_t)gu * P.capO * G, 0, cnt.x, pm, pinv, tid, nt);
  apply_pending<G>(P.qacc + (size_t)gu * P.capQ, P.qlg + (size_t)gu * P.capQ * G, 0, cnt.y, pm, pinv, tid, nt);
}

template <int D, int G, int BITS>
static hipError_t launch_decode_t(const Pools& P, const DecodeLaunch& a, hipStream_t s, hipEvent_t ev0,
                                  hipEvent_t ev1) {
  dim3 grid(a.splits, a.n_units);
  if (ev0) (void)hipEventRecord(ev0, s);
  hipLaunchKernelGGL((k_decode_attend<D, G, BITS>), grid, dim3(256), 0, s, P, a);
  if (ev1) (void)hipEventRecord(ev1, s);
  hipLaunchKernelGGL((k_decode_combine<D, G>), dim3(a.n_units), dim3(256), 0, s, P, a);
  return hipGetLastError();
}

template <int D, int G>
static hipError_t launch_decode_b(const Pools& P, const DecodeLaunch& a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
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

hipError_t launch_flush_scores(const Pools& P, int unit_begin, int n_units, int parity, hipStream_t s) {
  const int cap = P.capO > P.capQ ? P.capO : P.capQ;
  int bx = (cap + 255) / 256;
  if (bx > 32) bx = 32;
  dim3 grid(bx, n_units);
  switch (P.G) {
    case 1: hipLaunchKernelGGL((k_flush_scores<1>), grid, dim3(256), 0, s, P, unit_begin, parity); break;
    case 2: hipLaunchKernelGGL((k_flush_scores<2>), grid, dim3(256), 0, s, P, unit_begin, parity); break;
    case 4: hipLaunchKernelGGL((k_flush_scores<4>), grid, dim3(256), 0, s, P, unit_begin, parity); break;
    case 8: hipLaunchKernelGGL((k_flush_scores<8>), grid, dim3(256), 0, s, P, unit_begin, parity); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace arkv
