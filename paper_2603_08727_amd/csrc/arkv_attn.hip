// Causal prefill attention with the scorer's first pass fused (Sec. IV-C: eq. 2 is a slice of the prompt's
// causal attention, so the pass that computes the prompt's outputs already holds the window rows' softmax
// maxima and sums).
//
// One workgroup = 32 query positions of one (sequence, kv-head); wave w = q-head w of the group, so the G
// heads of a group share every key and value tile.  Keys are on the M side of the logits MFMA
// (v_mfma_f32_32x32x16_bf16, S^T = K Q^T), which leaves ONE query row per lane: the online softmax is
// per-lane arithmetic plus one exchange between the two lane halves.  The probabilities a lane then holds
// (keys 8(i/4) + 4(lane/32) + i%4 of the tile) are, eight at a time, exactly a B operand of the PV MFMA
// (O^T = V^T P^T) if the contraction index is read in that key order; the value tile is staged in LDS
// transposed ([channel][key], fp16) so that the matching A operand is two 8-byte reads.  Probabilities
// are rounded to fp16 (values to fp16 exactly or nearly: bf16 has fewer mantissa bits), accumulation fp32.
#include <hip/hip_fp16.h>

#include "arkv_dev.h"

namespace arkv {

typedef __bf16 bf16x8a __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8a __attribute__((ext_vector_type(8)));
typedef float f32x16a __attribute__((ext_vector_type(16)));

constexpr float kNegBigA = -1.0e30f;
constexpr int kVtPitch = 36;   // halves per channel row of the transposed value tile (32 keys + pad, 8-byte aligned)

__device__ __forceinline__ float aexp2(float x) { return __builtin_amdgcn_exp2f(x); }

// bf16 pair (low, high halves of a dword) -> fp16 pair
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t v) {
  const float lo = __uint_as_float(v << 16), hi = __uint_as_float(v & 0xffff0000u);
  const __half2 h = __floats2half2_rn(lo, hi);
  return *reinterpret_cast<const uint32_t*>(&h);
}

template <int D, int G>
__global__ __launch_bounds__(64 * G) void k_prefill_attn(AttnLaunch L) {
  constexpr int KK = D / 16;          // k-steps of the logits MFMA
  constexpr int CBN = D / 32;         // 32-channel blocks of the output
  constexpr int NT = 64 * G;
  __shared__ __align__(16) _Float16 vt[2][D][kVtPitch];
  const int qb = gridDim.x - 1 - blockIdx.x;      // long rows first
  const int u = blockIdx.y, b = u / L.Hkv, g = u % L.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = lane & 31, hh = lane >> 5;
  const int T = L.T, Tq = L.Tq, q0 = T - Tq;
  const int row = 32 * qb + n;                     // query row inside the block of T_q queries
  const int rowc_ = row < Tq ? row : Tq - 1;
  const int pos = q0 + rowc_;                      // its position: sees keys j <= pos
  const int jmax = min(T, q0 + 32 * qb + 32);      // keys any row of this workgroup can see
  const int ntiles = (jmax + 31) / 32;
  const uint16_t* kbase = L.k + (size_t)u * T * D;
  const uint16_t* vbase = L.v + (size_t)u * T * D;

  // query operand (B of S^T = K Q^T): row n, channels 16 kk + 8 hh .. +7
  uint4 qreg[KK];
  {
    const uint16_t* qp = L.q + ((size_t)(b * L.Hq + g * G + w) * Tq + rowc_) * D + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qreg[kk] = *reinterpret_cast<const uint4*>(qp + 16 * kk);
  }
  auto load_k = [&](uint4 (&kf)[KK], int j0) {
    const int key = min(j0 + n, T - 1);
    const uint16_t* p = kbase + (size_t)key * D + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = *reinterpret_cast<const uint4*>(p + 16 * kk);
  };
  // value tile: 32 keys x D channels = 4 D uint4 chunks, spread over the workgroup
  constexpr int VCH = 4 * D;                       // chunks of 8 channels
  constexpr int VPT = (VCH + NT - 1) / NT;         // chunks per thread
  auto load_v = [&](uint4 (&vr)[VPT], int j0) {
#pragma unroll
    for (int c = 0; c < VPT; ++c) {
      const int ch = min(tid + NT * c, VCH - 1);
      const int key = min(j0 + ch / (D / 8), T - 1);
      vr[c] = *reinterpret_cast<const uint4*>(vbase + (size_t)key * D + 8 * (ch % (D / 8)));
    }
  };
  auto stage_v = [&](const uint4 (&vr)[VPT], int buf) {
#pragma unroll
    for (int c = 0; c < VPT; ++c) {
      const int ch = tid + NT * c;
      if (ch < VCH) {
        const int key = ch / (D / 8), c0 = 8 * (ch % (D / 8));
        const uint32_t h[4] = {bf16x2_to_f16x2(vr[c].x), bf16x2_to_f16x2(vr[c].y), bf16x2_to_f16x2(vr[c].z),
                               bf16x2_to_f16x2(vr[c].w)};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          reinterpret_cast<uint16_t&>(vt[buf][c0 + 2 * e][key]) = (uint16_t)(h[e] & 0xffffu);
          reinterpret_cast<uint16_t&>(vt[buf][c0 + 2 * e + 1][key]) = (uint16_t)(h[e] >> 16);
        }
      }
    }
  };

  f32x16a acc[CBN];
#pragma unroll
  for (int cb = 0; cb < CBN; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;
  float m_run = kNegBigA, l_run = 0.f;

  uint4 kf[KK], kn[KK], vr[VPT];
  load_k(kf, 0);
  load_v(vr, 0);
  stage_v(vr, 0);
  __syncthreads();
  for (int t = 0; t < ntiles; ++t) {
    const int j0 = 32 * t, buf = t & 1;
    load_k(kn, j0 + 32);                            // clamped past the end
    load_v(vr, j0 + 32);
    f32x16a C;
#pragma unroll
    for (int i = 0; i < 16; ++i) C[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      C = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8a, kf[kk]), __builtin_bit_cast(bf16x8a, qreg[kk]), C, 0, 0, 0);
    // logits of row n against keys j0 + 8(i/4) + 4hh + i%4
    float x[16];
    float mt = kNegBigA;
    const bool need_mask = j0 + 31 > q0 + 32 * qb;   // some key of the tile is beyond some row of the block
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int j = j0 + 8 * (i >> 2) + 4 * hh + (i & 3);
      x[i] = (!need_mask || j <= pos) ? C[i] * L.scale2 : kNegBigA;
      mt = fmaxf(mt, x[i]);
    }
    mt = fmaxf(mt, __shfl_xor(mt, 32));
    if (__any(mt > m_run + 8.0f)) {                 // move the reference maximum (rare after the first tiles)
      const float mn = fmaxf(m_run, mt);
      const float f = aexp2(m_run - mn);
      m_run = mn;
      l_run *= f;
#pragma unroll
      for (int cb = 0; cb < CBN; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[cb][i] *= f;
    }
    float p[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) { p[i] = aexp2(x[i] - m_run); l_run += p[i]; }   // masked: 2^(-1e30 - m) = 0
    // probabilities as fp16, eight per PV k-step: jj = 0 -> i = 0..7, jj = 1 -> i = 8..15
    uint32_t ph[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const __half2 h2 = __floats2half2_rn(p[2 * e], p[2 * e + 1]);
      ph[e] = *reinterpret_cast<const uint32_t*>(&h2);
    }
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const uint4 pb = make_uint4(ph[4 * jj], ph[4 * jj + 1], ph[4 * jj + 2], ph[4 * jj + 3]);
#pragma unroll
      for (int cb = 0; cb < CBN; ++cb) {
        // A = V^T: channel 32 cb + n, keys 16 jj + 4 hh + (0..3) and 16 jj + 8 + 4 hh + (0..3)
        const _Float16* vrow = &vt[buf][32 * cb + n][16 * jj + 4 * hh];
        const uint2 a0 = *reinterpret_cast<const uint2*>(vrow);
        const uint2 a1 = *reinterpret_cast<const uint2*>(vrow + 8);
        const uint4 va = make_uint4(a0.x, a0.y, a1.x, a1.y);
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8a, va), __builtin_bit_cast(f16x8a, pb), acc[cb], 0, 0, 0);
      }
    }
    stage_v(vr, buf ^ 1);                           // the other buffer was last read one iteration ago
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = kn[kk];
    __syncthreads();
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_tot;
  if (row < Tq) {
    uint16_t* op = L.out + ((size_t)(b * L.Hq + g * G + w) * Tq + row) * D;
#pragma unroll
    for (int cb = 0; cb < CBN; ++cb)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        uint16_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float val = acc[cb][4 * i4 + e] * inv;
          uint32_t bits = __float_as_uint(val);
          bits += 0x7fffu + ((bits >> 16) & 1u);      // round to nearest even (finite values)
          o[e] = (uint16_t)(bits >> 16);
        }
        *reinterpret_cast<uint2*>(op + 32 * cb + 8 * i4 + 4 * hh) =
            make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
      }
    // the scorer's row constant c = max + log2(sum) of the window rows (row index: head-major, W per head)
    if (L.rowc && hh == 0 && pos >= T - L.W)
      L.rowc[(size_t)u * L.MP + w * L.W + (pos - (T - L.W))] = m_run + log2f(l_tot);
  }
}

hipError_t launch_prefill_attn(const AttnLaunch& a, hipStream_t s) {
  const int U = a.B * a.Hkv, G = a.Hq / a.Hkv;
  dim3 grid((a.Tq + 31) / 32, U);
#define ARKV_AT(D_, G_) if (a.D == D_ && G == G_) { hipLaunchKernelGGL((k_prefill_attn<D_, G_>), grid, dim3(64 * G_), 0, s, a); return hipGetLastError(); }
  ARKV_AT(128, 1) ARKV_AT(128, 2) ARKV_AT(128, 4) ARKV_AT(128, 8)
  ARKV_AT(64, 1) ARKV_AT(64, 2) ARKV_AT(64, 4) ARKV_AT(64, 8)
#undef ARKV_AT
  return hipErrorInvalidValue;
}

}  // namespace arkv
