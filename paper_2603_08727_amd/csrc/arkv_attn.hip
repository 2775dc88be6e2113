// Causal prefill attention with the scorer's first pass fused (Sec. IV-C: eq. 2 is a slice of the prompt's
// causal attention, so the pass that computes the prompt's outputs already holds the window rows' softmax
// maxima and sums).
//
// One workgroup = 32 query positions of one (sequence, kv-head); wave w = q-head w of the group, so the G
// heads of a group share every key and value tile, which is fetched from HBM once per workgroup and staged
// in LDS (keys in three buffers, values in two, one barrier per 32-key tile).  Keys are on the M side of the
// logits MFMA (v_mfma_f32_32x32x16_bf16, S^T = K Q^T), which leaves ONE query row per lane: the online softmax
// is per-lane arithmetic (the two lane halves of a row talk only when the row's reference maximum moves, which
// is rare: see the step below).  The probabilities a lane then holds
// (keys 8(i/4) + 4(lane/32) + i%4 of the tile) are, eight at a time, exactly a B operand of the PV MFMA
// (O^T = V^T P^T) if the contraction index is read in that key order; the value tile is staged transposed
// ([channel][key], fp16) with its key columns permuted so that the matching A operand is one 16-byte read.
// Probabilities are rounded to fp16 (values to fp16 exactly: bf16 has fewer mantissa bits; magnitudes
// beyond fp16's range are not supported), accumulation fp32.
#include <hip/hip_fp16.h>

#include "arkv_dev.h"

namespace arkv {

typedef __bf16 bf16x8a __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8a __attribute__((ext_vector_type(8)));
typedef float f32x16a __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4a __attribute__((ext_vector_type(4)));   // a 16-byte chunk the compiler keeps in registers

constexpr float kNegBigA = -1.0e30f;
constexpr int kVtPitch = 40;   // halves per channel row of the transposed value tile: 32 keys + 8 (16-byte reads, 20-dword stride)

__device__ __forceinline__ float aexp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two bf16 values (each in the LOW half of its dword) -> packed fp16 pair (a low, b high)
__device__ __forceinline__ uint32_t bf16_pair_to_f16x2(uint32_t a, uint32_t b) {
  const __half2 h = __floats2half2_rn(__uint_as_float(a << 16), __uint_as_float(b << 16));
  return *reinterpret_cast<const uint32_t*>(&h);
}

// column of key j (0..31) in the transposed value tile: the eight keys 16 jj + 8 a + 4 hh + r (a = 0, 1;
// r = 0..3) that lane half hh contracts in PV step jj sit side by side at 16 jj + 8 hh + 4 a + r
__device__ __forceinline__ int vt_col(int j) { return (j & 16) | ((j & 4) << 1) | ((j & 8) >> 1) | (j & 3); }

template <int D>
struct AttnLds {
  static constexpr int KP = D + 8;              // halves per key row: 16-byte reads of 16 keys hit 64 banks
  uint16_t k[3][32][KP];                        // key tiles t + 1 (logits now), t + 2 (operands prefetched), t + 3 (being staged)
  _Float16 vt[2][D][kVtPitch];
};

// sched_group_barrier classes
constexpr int kSgValu = 0x2, kSgMfma = 0x8, kSgDsRead = 0x100;
typedef _Float16 f16x2a __attribute__((ext_vector_type(2)));
constexpr float kSumLimit = 16384.0f;   // a lane's 16 probabilities may sum to this before the reference maximum moves

// Profiling builds (-DARKV_PHASE_TRACE): shader-clock and 100 MHz timestamps around the longest workgroup,
// from which the shader clock the kernel ran at follows.  Product builds compile none of it.
#ifdef ARKV_PHASE_TRACE
__device__ unsigned long long g_attn_clock[4];
#endif

template <int D, int G>
__global__ __launch_bounds__(64 * G, G >= 4 ? 2 : 1) void k_prefill_attn(AttnLaunch L) {
#ifdef ARKV_PHASE_TRACE
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) { g_attn_clock[0] = clock64(); g_attn_clock[1] = wall_clock64(); }
#endif
  constexpr int KK = D / 16;          // k-steps of the logits MFMA
  constexpr int KH = KK / 2;          // operands carried from the previous phase
  constexpr int CBN = D / 32;         // 32-channel blocks of the output
  constexpr int NPV = 2 * CBN;        // PV MFMAs per tile
  constexpr int NT = 64 * G;
  constexpr int CPR = D / 8;          // 16-byte chunks per row
  constexpr int KCH = 32 * CPR;       // key chunks per tile
  constexpr int VCH = 16 * CPR;       // value chunk pairs (two adjacent keys, eight channels) per tile
  constexpr int KPT = (KCH + NT - 1) / NT;
  constexpr int VPT = (VCH + NT - 1) / NT;
  static_assert(NPV >= KH, "operand prefetch pattern");
  __shared__ __align__(16) AttnLds<D> sm;
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
  const int jfull = q0 + 32 * qb - 31;             // tiles starting at or before this need no mask
  const uint16_t* kbase = L.k + (size_t)u * T * D;
  const uint16_t* vbase = L.v + (size_t)u * T * D;
  const float scale2 = L.scale2;

  // query operand (B of S^T = K Q^T): row n, channels 16 kk + 8 hh .. +7
  u32x4a qreg[KK];
  {
    const uint16_t* qp = L.q + ((size_t)(b * L.Hq + g * G + w) * Tq + rowc_) * D + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qreg[kk] = *reinterpret_cast<const u32x4a*>(qp + 16 * kk);
  }
  // global -> registers -> LDS staging of one tile.  A tile that ends inside the prompt is addressed as a
  // uniform base plus a per-thread constant; the last, partial one (and the prefetch past it) clamps its rows
  // to the prompt: the surplus keys are masked or never read.
  u32x4a ks[KPT], vs[VPT][2];
  auto fetch_k = [&](int j0) {
    if (j0 + 32 <= T) {
      const uint16_t* base = kbase + (size_t)j0 * D;
#pragma unroll
      for (int c = 0; c < KPT; ++c) {
        const int ch = min(tid + NT * c, KCH - 1);
        ks[c] = *reinterpret_cast<const u32x4a*>(base + (ch / CPR) * D + 8 * (ch % CPR));
      }
    } else {
#pragma unroll
      for (int c = 0; c < KPT; ++c) {
        const int ch = min(tid + NT * c, KCH - 1);
        const int key = min(j0 + ch / CPR, T - 1);
        ks[c] = *reinterpret_cast<const u32x4a*>(kbase + (size_t)key * D + 8 * (ch % CPR));
      }
    }
  };
  auto fetch_v = [&](int j0) {
    if (j0 + 32 <= T) {
      const uint16_t* base = vbase + (size_t)j0 * D;
#pragma unroll
      for (int c = 0; c < VPT; ++c) {
        const int ch = min(tid + NT * c, VCH - 1);
        const uint16_t* p = base + 2 * (ch % 16) * D + 8 * (ch / 16);
        vs[c][0] = *reinterpret_cast<const u32x4a*>(p);
        vs[c][1] = *reinterpret_cast<const u32x4a*>(p + D);
      }
    } else {
#pragma unroll
      for (int c = 0; c < VPT; ++c) {
        const int ch = min(tid + NT * c, VCH - 1);
        const int k0 = min(j0 + 2 * (ch % 16), T - 1), k1 = min(j0 + 2 * (ch % 16) + 1, T - 1);
        vs[c][0] = *reinterpret_cast<const u32x4a*>(vbase + (size_t)k0 * D + 8 * (ch / 16));
        vs[c][1] = *reinterpret_cast<const u32x4a*>(vbase + (size_t)k1 * D + 8 * (ch / 16));
      }
    }
  };
  auto stage_k = [&](int buf) {
#pragma unroll
    for (int c = 0; c < KPT; ++c) {
      const int ch = tid + NT * c;
      if (KCH % NT == 0 || ch < KCH) *reinterpret_cast<u32x4a*>(&sm.k[buf][ch / CPR][8 * (ch % CPR)]) = ks[c];
    }
  };
  auto stage_v = [&](int buf) {
#pragma unroll
    for (int c = 0; c < VPT; ++c) {
      const int ch = tid + NT * c;
      if (VCH % NT == 0 || ch < VCH) {
        const int col = vt_col(2 * (ch % 16)), c0 = 8 * (ch / 16);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          *reinterpret_cast<uint32_t*>(&sm.vt[buf][c0 + 2 * e][col]) = bf16_pair_to_f16x2(vs[c][0][e], vs[c][1][e]);
          *reinterpret_cast<uint32_t*>(&sm.vt[buf][c0 + 2 * e + 1][col]) = bf16_pair_to_f16x2(vs[c][0][e] >> 16, vs[c][1][e] >> 16);
        }
      }
    }
  };
  auto k_operand = [&](int buf, int kk) { return *reinterpret_cast<const u32x4a*>(&sm.k[buf][n][16 * kk + 8 * hh]); };
  // A of O^T = V^T P^T, PV MFMA r = jj * CBN + cb: channel 32 cb + n, keys 16 jj + 4 hh + (0..3) and
  // 16 jj + 8 + 4 hh + (0..3), adjacent in LDS
  auto v_operand = [&](int buf, int r) {
    return *reinterpret_cast<const u32x4a*>(&sm.vt[buf][32 * (r % CBN) + n][16 * (r / CBN) + 8 * hh]);
  };

  f32x16a acc[CBN];
#pragma unroll
  for (int cb = 0; cb < CBN; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;
  float m_run = kNegBigA, l_run = 0.f;
  u32x4a kop[KK], vop[NPV];
  int kA = 1, kB = 2, kW = 0;       // LDS buffers of key tiles t + 1, t + 2 and t + 3 (= the one tile t leaves)

  // fresh logits of the tile starting at j0 (C[i]: row n against key j0 + 8(i/4) + 4hh + i%4, unscaled):
  // what lies beyond the row gets a logit whose probability is zero
  auto mask = [&](f32x16a& C, int j0) {
    if (j0 > jfull) {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (j0 + 8 * (i >> 2) + 4 * hh + (i & 3) > pos) C[i] = kNegBigA;
    }
  };
  // probabilities of logits C against the running reference m_run, as fp16 pairs (ph[e]: elements 2e, 2e + 1),
  // and their sum as rounded (the same numbers the PV MFMA multiplies)
  auto probs = [&](const f32x16a& C, int i, uint32_t (&ph)[8], float& lt) {
    const float p0 = aexp2(fmaf(C[i], scale2, -m_run)), p1 = aexp2(fmaf(C[i + 1], scale2, -m_run));
    const __half2 h2 = __floats2half2_rn(p0, p1);
    ph[i / 2] = *reinterpret_cast<const uint32_t*>(&h2);
    lt = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2a, ph[i / 2]), f16x2a{(_Float16)1.0f, (_Float16)1.0f}, lt, false);
  };

  // One step of the two-stage pipeline over tiles.  Phase A: the logits MFMAs of tile t + 1 (into Cn), each
  // followed in issue order by one LDS operand read for a later MFMA and by its share of tile t's softmax
  // arithmetic (from C): the matrix pipe works in the background of the same wave's vector instructions only
  // if the two alternate.  Phase B: the PV MFMAs of tile t between operand reads for the next step and the
  // conversion of the tiles fetched at the top, which are staged into LDS at the end.
  // The reference maximum is lazy: probabilities are taken against the row's current m_run, and only when a
  // lane's sum shows that they grew large (or the reference is still unset) does the row move its reference
  // to the tile's maximum and redo the tile.  A row decides from its own numbers only.
  auto step = [&](f32x16a& C, f32x16a& Cn, int t) {
    const int j0 = 32 * t, vb = t & 1;
    fetch_k(j0 + 96);
    fetch_v(j0 + 32);
    uint32_t ph[8];
    float lt0 = 0.f, lt1 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) Cn[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk + KH < KK) kop[kk + KH] = k_operand(kA, kk + KH);
      else vop[kk + KH - KK] = v_operand(vb, kk + KH - KK);
      Cn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8a, kop[kk]), __builtin_bit_cast(bf16x8a, qreg[kk]), Cn, 0, 0, 0);
      constexpr int EPK = 16 / KK;                    // softmax elements per MFMA (2 at D = 128, 4 at D = 64)
#pragma unroll
      for (int e = 0; e < EPK; e += 2) probs(C, EPK * kk + e, ph, ((kk + e / 2) & 1) ? lt1 : lt0);
    }
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_group_barrier(kSgMfma, 1, 0);
      __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
      __builtin_amdgcn_sched_group_barrier(kSgValu, 6 * 16 / (2 * KK), 0);
    }
    float lt = lt0 + lt1;
    if (__any(!(lt <= kSumLimit))) {                  // rare after the first tile
      const float lo = __shfl_xor(lt, 32);
      const bool move = !(fmaxf(lt, lo) <= kSumLimit);   // both lane halves of a row agree
      float mt = C[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mt = fmaxf(mt, C[i]);
      mt *= scale2;                                   // scale2 > 0: the maximum commutes with the scaling
      mt = fmaxf(mt, __shfl_xor(mt, 32));
      const float mn = move ? fmaxf(m_run, mt) : m_run;
      const float f = aexp2(m_run - mn);
      m_run = mn;
      l_run *= f;
#pragma unroll
      for (int cb = 0; cb < CBN; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[cb][i] *= f;
      lt0 = 0.f; lt1 = 0.f;
#pragma unroll
      for (int i = 0; i < 16; i += 2) probs(C, i, ph, lt0);
      lt = lt0;
    }
    l_run += lt;
    // PV: probabilities eight per k-step: jj = 0 -> elements 0..7, jj = 1 -> 8..15
#pragma unroll
    for (int r = 0; r < NPV; ++r) {
      if (r + KH < NPV) vop[r + KH] = v_operand(vb, r + KH);
      else kop[r + KH - NPV] = k_operand(kB, r + KH - NPV);
      const int jj = r / CBN, cb = r % CBN;
      const u32x4a pb = {ph[4 * jj], ph[4 * jj + 1], ph[4 * jj + 2], ph[4 * jj + 3]};
      acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8a, vop[r]), __builtin_bit_cast(f16x8a, pb), acc[cb], 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < NPV; ++r) {
      __builtin_amdgcn_sched_group_barrier(kSgMfma, 1, 0);
      __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);                // the staging waits for this step's loads: keep it behind the MFMAs
    stage_k(kW);                                      // tile t + 3 into the buffer tile t's logits came from
    stage_v(vb ^ 1);                                  // tile t + 1; that buffer was last read one step ago
    mask(Cn, j0 + 32);
    const int k0 = kA; kA = kB; kB = kW; kW = k0;
    __syncthreads();
  };

  fetch_k(0);
  fetch_v(0);
  stage_k(0);
  stage_v(0);
  fetch_k(32);
  stage_k(1);
  fetch_k(64);
  stage_k(2);
  __syncthreads();
  f32x16a C0, C1;
  {
#pragma unroll
    for (int i = 0; i < 16; ++i) C0[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      C0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8a, k_operand(0, kk)), __builtin_bit_cast(bf16x8a, qreg[kk]), C0, 0, 0, 0);
    mask(C0, 0);
#pragma unroll
    for (int kk = 0; kk < KH; ++kk) kop[kk] = k_operand(1, kk);
  }
  for (int t = 0; t < ntiles; t += 2) {
    step(C0, C1, t);
    if (t + 1 < ntiles) step(C1, C0, t + 1);
  }

#ifdef ARKV_PHASE_TRACE
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) { g_attn_clock[2] = clock64(); g_attn_clock[3] = wall_clock64(); }
#endif
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_tot;
  if (row < Tq) {
    uint16_t* op = L.out + ((size_t)(b * L.Hq + g * G + w) * Tq + row) * D;
    float* opf = L.outf ? L.outf + ((size_t)(b * L.Hq + g * G + w) * Tq + row) * D : nullptr;   // parity hook
#pragma unroll
    for (int cb = 0; cb < CBN; ++cb)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        uint16_t o[4];
        float of[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float val = acc[cb][4 * i4 + e] * inv;
          of[e] = val;
          uint32_t bits = __float_as_uint(val);
          bits += 0x7fffu + ((bits >> 16) & 1u);      // round to nearest even (finite values)
          o[e] = (uint16_t)(bits >> 16);
        }
        if (opf) *reinterpret_cast<float4*>(opf + 32 * cb + 8 * i4 + 4 * hh) = make_float4(of[0], of[1], of[2], of[3]);
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

namespace arkv {
// the prefill attention's four clock words (shader clock and 100 MHz counter at the start and the end of workgroup 0)
hipError_t phase_trace_attn(unsigned long long* host, bool* built) {
#ifdef ARKV_PHASE_TRACE
  *built = true;
  return hipMemcpyFromSymbol(host, HIP_SYMBOL(g_attn_clock), 4 * sizeof(unsigned long long));
#else
  (void)host;
  *built = false;
  return hipSuccess;
#endif
}
}  // namespace arkv
