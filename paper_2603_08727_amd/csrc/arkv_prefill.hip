// Prefill scorer (Sec. IV-C eqs. 2-5, and the first samples of the eq. 9 moments).
//
// Per unit (sequence, kv-head) the last W queries of the G heads of the group form M = G*W query
// rows; their logits against all T keys are a dense [T x d] x [d x M] contraction -> MFMA
// (v_mfma_f32_32x32x16_bf16, keys on the M side so that a lane owns ONE query row and the softmax
// statistics of a row are in-register reductions).  The causal softmax needs each row's max and
// sum before any probability exists, so the keys are streamed twice:
//   k_prefill_rows     per (key chunk, unit): row max / row sum partials
//   k_prefill_rowfinal per unit: c_r = max_r + log2(sum_r)
//   k_prefill_cols     per (key chunk, unit): p = 2^(x - c_r); per key sum_r p and sum_r p^2 -> pre
//   k_prefill_stats    per sequence: p_k over keys < T-W aggregated over all heads, entropy,
//                      variance, kurtosis (fp64 reductions; the normaliser's partial sums come from
//                      k_prefill_cols, the last workgroup of a sequence finishes)
#include <type_traits>

#include "arkv_dev.h"

namespace arkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegBigP = -1.0e30f;

// 2^x as one v_exp_f32 (arguments are <= 0 up to rounding, or hugely negative -> 0)
__device__ __forceinline__ float pexp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CTRL>
__device__ __forceinline__ float dpp_p(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL,
                                                               0xf, 0xf, true));
}
// sum over the 32 lanes that share lane/32
__device__ __forceinline__ float sum32(float x) {
  x += dpp_p<0xB1>(x);
  x += dpp_p<0x4E>(x);
  x += dpp_p<0x141>(x);
  x += dpp_p<0x140>(x);
  x += __shfl_xor(x, 16);
  return x;
}

// Stage the unit's query rows in LDS: row r = (head r / W, window query r % W) at byte r*(2D+16), rows >= M
// zero.  q points at the unit's first head; heads are head_stride elements apart.
template <int D, int NT>
__device__ __forceinline__ void stage_q(unsigned char* sm, const uint16_t* q, size_t head_stride, int W, int M, int MP) {
  constexpr int RB = 2 * D + 16;
  constexpr int VPR = D / 8;  // uint4 per row
  constexpr int BATCH = 8;    // loads in flight per thread (one at a time, every load costs a memory round trip)
  for (int i0 = threadIdx.x; i0 < MP * VPR; i0 += NT * BATCH) {
    uint4 v[BATCH];
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
      const int i = i0 + b * NT, r = i / VPR, c = i % VPR;
      v[b] = make_uint4(0, 0, 0, 0);
      if (r < M) v[b] = *reinterpret_cast<const uint4*>(q + (size_t)(r / W) * head_stride + (size_t)(r % W) * D + c * 8);
    }
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
      const int i = i0 + b * NT, r = i / VPR, c = i % VPR;
      if (i < MP * VPR) *reinterpret_cast<uint4*>(sm + (size_t)r * RB + c * 16) = v[b];
    }
  }
}

template <int D>
__device__ __forceinline__ void load_keys(u32x4 (&kf)[D / 16], const uint16_t* k, int j0, int T, int lane) {
  int key = j0 + (lane & 31);
  if (key > T - 1) key = T - 1;
  const uint16_t* p = k + (size_t)key * D + (lane >> 5) * 8;
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) kf[kk] = *reinterpret_cast<const u32x4*>(p + kk * 16);
}

// One step of the two passes' software pipeline: the D/16 MFMAs that form the NEXT step's 32x32 logits tile
// (key operands kx, query operands of row tile rt_next read from LDS two MFMAs ahead), with the vector work on
// THIS step's tile dealt out between them by `work(kk)`.  A wave's MFMAs only run in the background of its own
// vector instructions if the two alternate in the instruction stream, and left to itself the compiler groups
// them apart (scheduling barriers do not help: the instruction selector has already grouped them).  The order is
// therefore pinned by data: after slot kk an empty volatile asm takes the two running sums of the vector work
// (p0, p1: every slot's work must read and write them) together with the key operand of MFMA kk + 1, so that
// work(kk) lies before it and MFMA kk + 1 after it.
// KEYS_ON_M: the keys are the MFMA's M side (a lane owns one query row), else its N side (a lane owns one key).
// qoff: the lane's byte offset inside a row tile, (lane % 32) * row pitch + (lane / 32) * 16; it goes through an
// empty asm so that the optimiser cannot hoist the LDS reads (the same for every key tile) out of the key loop,
// where they would take 32 RT registers.
// LDS operands are requested this many MFMAs ahead, across steps (a whole step ahead measured the same and costs
// 16 registers more)
template <int D> constexpr int kQAheadOf = 3;

// The first kQAhead operands of row tile rt: what a step expects to be in flight when it starts.
template <int D>
__device__ __forceinline__ void prime_operands(uint4 (&qb)[kQAheadOf<D> + 1], const unsigned char* sm, int rt, int qoff) {
  constexpr int RB = 2 * D + 16;
  constexpr int kQAhead = kQAheadOf<D>;
  asm volatile("" : "+v"(qoff));
#pragma unroll
  for (int i = 0; i < kQAhead; ++i) qb[i] = *reinterpret_cast<const uint4*>(sm + rt * 32 * RB + qoff + i * 32);
}

// rt_next: the row tile whose logits this step's MFMAs form; rt_after: the row tile of the step after it, whose
// first kQAhead operands are requested in this step's last slots (ring qb, slot = operand index % (kQAhead + 1);
// D/16 is a multiple of the ring size, so the slots line up from step to step).
template <int D, bool KEYS_ON_M, typename Work>
__device__ __forceinline__ f32x16 pipeline_step(u32x4 (&kx)[D / 16], uint4 (&qb)[kQAheadOf<D> + 1], const unsigned char* sm,
                                                int rt_next, int rt_after, int qoff, float& p0, float& p1, Work work) {
  constexpr int RB = 2 * D + 16;
  constexpr int KK = D / 16;
  constexpr int kQAhead = kQAheadOf<D>;
  static_assert(KK % (kQAhead + 1) == 0 && KK > kQAhead, "ring slots must line up across steps");
  asm volatile("" : "+v"(qoff));
  const unsigned char* qrow = sm + rt_next * 32 * RB + qoff;
  const unsigned char* qrow2 = sm + rt_after * 32 * RB + qoff;
  f32x16 C = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    const int ahead = kk + kQAhead;
    qb[ahead % (kQAhead + 1)] = *reinterpret_cast<const uint4*>(ahead < KK ? qrow + ahead * 32 : qrow2 + (ahead - KK) * 32);
    const uint4 qc = qb[kk % (kQAhead + 1)];
    if constexpr (KEYS_ON_M)
      C = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kx[kk]), __builtin_bit_cast(bf16x8, qc), C, 0, 0, 0);
    else
      C = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, qc), __builtin_bit_cast(bf16x8, kx[kk]), C, 0, 0, 0);
    work(kk);
    if (kk + 1 < KK) {
      // (resident since the previous key tile: pinning it waits for nothing)
      asm volatile("" : "+v"(p0), "+v"(p1), "+v"(kx[kk + 1]));
    }
  }
  return C;
}

// NW waves per workgroup: 4, or 8 where the staged queries leave room for only one workgroup per CU (more than
// 256 query rows), so that a SIMD still has two waves.
// Logits tile of the first pass: C[i] at key j0 + 8(i/4) + 4(lane/32) + i%4, row rt*32 + lane%32.
template <int D, int RT, int NW>
__global__ __launch_bounds__(64 * NW, (NW == 4 && RT < 8) ? 3 : 2) void k_prefill_rows(PrefillLaunch L) {
  extern __shared__ __align__(16) unsigned char sm[];
  constexpr int NT = 64 * NW;
  constexpr int KK = D / 16;
  const int chunk = blockIdx.x, u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int M = L.G * L.W, MP = RT * 32, T = L.T;
  stage_q<D, NT>(sm, L.q_win + (size_t)u * L.G * L.q_head_stride, L.q_head_stride, L.W, M, MP);
  __syncthreads();
  const uint16_t* k = L.k + (size_t)u * T * D;
  float m[RT], l[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) { m[rt] = kNegBigP; l[rt] = 0.f; }
  const int jbeg = chunk * L.chunk, jend = min(jbeg + L.chunk, T);
  const int qoff = (lane & 31) * (2 * D + 16) + (lane >> 5) * 16;
  const float scale2 = L.scale2;
  u32x4 kf[KK], kn[KK];
  if (jbeg + w * 32 < jend) load_keys<D>(kf, k, jbeg + w * 32, T, lane);
  float pin0 = 0.f, pin1 = 0.f;
  uint4 qb[kQAheadOf<D> + 1];
  prime_operands<D>(qb, sm, 0, qoff);
  f32x16 C = pipeline_step<D, true>(kf, qb, sm, 0, RT > 1 ? 1 : 0, qoff, pin0, pin1, [](int) {});
  // One key tile against all row tiles; every step also issues the next step's MFMAs.  FULL: no key of the tile
  // is masked for any row (padded rows are rows of zeros whose statistics nobody reads), and then nothing in the
  // body branches.
  auto key_tile = [&](int j0, auto full_c) {
    constexpr bool FULL = decltype(full_c)::value;
    load_keys<D>(kn, k, j0 + 32 * NW, T, lane);        // next tile of this wave (clamped past the end)
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      float x[16];
      float mn = 0.f, s = 0.f;
      auto work = [&](int kk) {
        if (kk == 0) {
          if constexpr (FULL) {
            // the scale is positive, so the maximum is taken on the raw dot products
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = C[i];
            float mt = fmaxf(x[0], x[1]);
#pragma unroll
            for (int i = 2; i < 16; i += 2) mt = fmaxf(fmaxf(mt, x[i]), x[i + 1]);
            mn = fmaxf(m[rt], mt * scale2);
          } else {
            const int r = rt * 32 + (lane & 31);
            const int lastv = r < M ? T - L.W + (r % L.W) : -1;   // last visible key of this row
            float mt = kNegBigP;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int j = j0 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
              x[i] = j <= lastv ? C[i] * scale2 : kNegBigP;       // scaled here: the sentinel stays the sentinel
              mt = fmaxf(mt, x[i]);
            }
            mn = fmaxf(m[rt], mt);
          }
          s = l[rt] * pexp2(m[rt] - mn);
        } else {
          // the 16 logits are dealt over the remaining KK - 1 slots; FULL: 2^(scale x - max) is one fma and one exp
          const int i0 = (kk - 1) * 16 / (KK - 1), i1 = kk * 16 / (KK - 1);
#pragma unroll
          for (int i = i0; i < i1; ++i) {
            if constexpr (FULL) s += pexp2(fmaf(x[i], scale2, -mn));
            else s += pexp2(x[i] - mn);                           // masked entries: 2^(-1e30 - mn) = 0
          }
        }
      };
      constexpr int RT2 = RT > 1 ? 1 : 0;          // the row tile after row tile 0
      const f32x16 Cn = rt + 1 < RT ? pipeline_step<D, true>(kf, qb, sm, rt + 1, rt + 2 < RT ? rt + 2 : 0, qoff, mn, s, work)
                                    : pipeline_step<D, true>(kn, qb, sm, 0, RT2, qoff, mn, s, work);
      if constexpr (!FULL) { if (!(mn > 0.5f * kNegBigP)) s = 0.f; }      // nothing visible yet: 16 * 2^0 dropped
      m[rt] = mn; l[rt] = s;
      C = Cn;
    }
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = kn[kk];
  };
  int j0 = jbeg + w * 32;
  for (; j0 < jend && j0 + 32 <= T - L.W; j0 += 32 * NW) key_tile(j0, std::true_type{});
  for (; j0 < jend; j0 += 32 * NW) key_tile(j0, std::false_type{});
  // merge the two lane halves, then the waves
  float* red = reinterpret_cast<float*>(sm);   // reuse after everyone is done with the queries
  __syncthreads();
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const float mo = __shfl_xor(m[rt], 32), lo = __shfl_xor(l[rt], 32);
    const float mn = fmaxf(m[rt], mo);
    l[rt] = l[rt] * exp2f(m[rt] - mn) + lo * exp2f(mo - mn);
    m[rt] = mn;
    if (lane < 32) { red[(w * MP + rt * 32 + lane) * 2] = m[rt]; red[(w * MP + rt * 32 + lane) * 2 + 1] = l[rt]; }
  }
  __syncthreads();
  for (int r = tid; r < MP; r += NT) {
    float mn = kNegBigP;
    for (int i = 0; i < NW; ++i) mn = fmaxf(mn, red[(i * MP + r) * 2]);
    float s = 0.f;
    for (int i = 0; i < NW; ++i) s += red[(i * MP + r) * 2 + 1] * exp2f(red[(i * MP + r) * 2] - mn);
    L.rowstat[((size_t)u * L.n_chunks + chunk) * MP + r] = make_float2(mn, s);
  }
}

__global__ __launch_bounds__(256) void k_prefill_rowfinal(PrefillLaunch L, int MP, float* rowc) {
  // grid (MP/32, U): 32 rows per workgroup, 8 threads per row share the chunks
  __shared__ float sm_m[32][8], sm_s[32][8];
  const int u = blockIdx.y, r = blockIdx.x * 32 + (threadIdx.x >> 3), part = threadIdx.x & 7;
  float mn = kNegBigP;
  for (int c = part; c < L.n_chunks; c += 8) mn = fmaxf(mn, L.rowstat[((size_t)u * L.n_chunks + c) * MP + r].x);
  sm_m[threadIdx.x >> 3][part] = mn;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) mn = fmaxf(mn, sm_m[threadIdx.x >> 3][i]);
  float s = 0.f;
  for (int c = part; c < L.n_chunks; c += 8) {
    const float2 t = L.rowstat[((size_t)u * L.n_chunks + c) * MP + r];
    s += t.y * pexp2(t.x - mn);
  }
  sm_s[threadIdx.x >> 3][part] = s;
  __syncthreads();
  if (part == 0) {
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) tot += sm_s[threadIdx.x >> 3][i];
    rowc[(size_t)u * MP + r] = tot > 0.f ? mn + log2f(tot) : 0.f;
  }
}

__device__ __forceinline__ double block_sum_d(double v, double* sm) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[w] = v;
  __syncthreads();
  double t = 0;
  for (int i = 0; i < (int)(blockDim.x >> 6); ++i) t += sm[i];
  return t;
}

// Second pass.  Here the MFMA is turned round (query rows on the M side, keys on the N side) so that a
// lane owns ONE key and the sums over the M = G*W query rows are in-register additions: C[i] is row
// rt*32 + 8(i/4) + 4(lane/32) + i%4 against key j0 + lane%32.  The row constants c_r come from LDS.
template <int D, int RT, int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 3 : 2) void k_prefill_cols(PrefillLaunch L, const float* rowc, double* zpart) {
  extern __shared__ __align__(16) unsigned char sm[];
  constexpr int RB = 2 * D + 16;
  constexpr int NT = 64 * NW;
  constexpr int KK = D / 16;
  const int chunk = blockIdx.x, u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int M = L.G * L.W, MP = RT * 32, T = L.T;
  stage_q<D, NT>(sm, L.q_win + (size_t)u * L.G * L.q_head_stride, L.q_head_stride, L.W, M, MP);
  float* crow = reinterpret_cast<float*>(sm + (size_t)MP * RB);   // [MP] -c_r (padded rows: -1e30 -> p = 0)
  int* lastk = reinterpret_cast<int*>(crow + MP);                 // [MP] last visible key of the row
  for (int r = tid; r < MP; r += NT) {
    // the row constant in base-2 units: from the first pass / the attention pass, or from the caller's
    // log-sum-exp (natural log of the sum over visible keys of exp(scale q.k), what attention kernels commonly
    // return per query row; row r = (head inside the group) * W + (window query))
    float cr = 0.f;
    if (r < M) cr = L.lse ? L.lse[((size_t)u * L.G + r / L.W) * L.W + r % L.W] * 1.4426950408889634f : rowc[(size_t)u * MP + r];
    crow[r] = r < M ? -cr : kNegBigP;
    lastk[r] = r < M ? T - L.W + (r % L.W) : -1;
  }
  __syncthreads();
  const uint16_t* k = L.k + (size_t)u * T * D;
  const int jbeg = chunk * L.chunk, jend = min(jbeg + L.chunk, T);
  float2* pre = L.pre + (size_t)u * T;
  const int hl = lane >> 5, kl = lane & 31;
  const int qoff = kl * RB + hl * 16;
  const float scale2 = L.scale2;
  double zacc = 0.0;                                              // this workgroup's share of eq. 3's normaliser
  u32x4 kf[KK], kn[KK];
  if (jbeg + w * 32 < jend) load_keys<D>(kf, k, jbeg + w * 32, T, lane);
  float pin0 = 0.f, pin1 = 0.f;
  uint4 qb[kQAheadOf<D> + 1];
  prime_operands<D>(qb, sm, 0, qoff);
  f32x16 C = pipeline_step<D, false>(kf, qb, sm, 0, RT > 1 ? 1 : 0, qoff, pin0, pin1, [](int) {});
  float4 nc_nxt = *reinterpret_cast<const float4*>(crow + 4 * hl);      // row tile 0, first group
  // FULL: no key of the tile is masked for any row (padded rows have c_r = -1e30, so p = 0 without a test)
  auto key_tile = [&](int j0, auto full_c) {
    constexpr bool FULL = decltype(full_c)::value;
    load_keys<D>(kn, k, j0 + 32 * NW, T, lane);
    const int j = j0 + kl;
    float a1 = 0.f, a2 = 0.f;
    // the row constants are the same for every key tile too: opaque offset, see pipeline_step
    int c0 = 4 * hl;
    asm volatile("" : "+v"(c0));
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      // a slot handles PER logits: rows 8 g4 + 4 hl .. + 3 of the tile for g4 = first logit / 4.  The four row
      // constants of a group are requested from LDS one group ahead (nc_nxt; across steps and key tiles as well:
      // used right after the request, every group would wait for an LDS round trip)
      const int rt_n = rt + 1 < RT ? rt + 1 : 0;        // the tile the next step works on
      float4 nc;
      int4 lk;
      auto work = [&](int kk) {
        static_assert(KK == 8 || KK == 4, "two or four logits per slot");
        constexpr int PER = 16 / KK;                      // logits per slot
        const int i0 = kk * PER;
        if (i0 % 4 == 0) {
          const int g4 = i0 / 4;
          nc = nc_nxt;
          nc_nxt = *reinterpret_cast<const float4*>(crow + (g4 + 1 < 4 ? rt * 32 + 8 * (g4 + 1) : rt_n * 32) + c0);
          if constexpr (!FULL) lk = *reinterpret_cast<const int4*>(lastk + rt * 32 + 8 * g4 + c0);
        }
        const float ncv[4] = {nc.x, nc.y, nc.z, nc.w};
        const int lkv[4] = {lk.x, lk.y, lk.z, lk.w};
#pragma unroll
        for (int i = i0; i < i0 + PER; ++i) {
          float p = pexp2(fmaf(C[i], scale2, ncv[i % 4]));
          if constexpr (!FULL) p = j <= lkv[i % 4] ? p : 0.f;
          a1 += p;
          a2 = fmaf(p, p, a2);
        }
      };
      constexpr int RT2 = RT > 1 ? 1 : 0;          // the row tile after row tile 0
      const f32x16 Cn = rt + 1 < RT ? pipeline_step<D, false>(kf, qb, sm, rt + 1, rt + 2 < RT ? rt + 2 : 0, qoff, a1, a2, work)
                                    : pipeline_step<D, false>(kn, qb, sm, 0, RT2, qoff, a1, a2, work);
      C = Cn;
    }
    a1 += __shfl_xor(a1, 32);
    a2 += __shfl_xor(a2, 32);
    if (hl == 0 && j < T) pre[j] = make_float2(a1, a2);
    if (hl == 0 && j < T - L.W) zacc += (double)a1;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = kn[kk];
  };
  int j0 = jbeg + w * 32;
  for (; j0 < jend && j0 + 32 <= T - L.W; j0 += 32 * NW) key_tile(j0, std::true_type{});
  for (; j0 < jend; j0 += 32 * NW) key_tile(j0, std::false_type{});
  // sum over the chunk's keys before the window of the attention they received, in a fixed order
  zacc = block_sum_d(zacc, reinterpret_cast<double*>(sm));       // (its first barrier ends the use of the queries)
  if (tid == 0) zpart[(size_t)u * L.n_chunks + chunk] = zacc;
}

// Results that one workgroup writes and another reads inside the same launch go through device-scope relaxed
// atomics (write-through stores, loads that do not hit a stale L2 line of another XCD); no cache-wide flush.
__device__ __forceinline__ void st_dev_d(double* p, double v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ double ld_dev_d(const double* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Aggregated key distribution over ALL heads of a sequence and its three statistics (eqs. 3-5), fp64, every
// sum in a fixed order: the normaliser Z from the column pass's per-workgroup sums; per chunk of keys the sums
// of -p ln p, (p - 1/n)^2, (p - 1/n)^4; the workgroup of a sequence that finishes last (a ticket) adds the
// chunks up and writes the statistics.
constexpr int kStatChunk = 512;    // keys per workgroup

__global__ __launch_bounds__(256) void k_prefill_stats(PrefillLaunch L, const double* zpart, double* mpart) {
  __shared__ double sm[16];
  __shared__ int last;
  const int b = blockIdx.y, ch = blockIdx.x, n = L.T - L.W, nch = gridDim.x;
  const float2* pre = L.pre + (size_t)b * L.Hkv * L.T;
  double Z = 0;
  for (int i = threadIdx.x; i < L.Hkv * L.n_chunks; i += 256) Z += zpart[(size_t)b * L.Hkv * L.n_chunks + i];
  Z = block_sum_d(Z, sm);
  const double pbar = 1.0 / (double)n;
  const int j1 = min(n, (ch + 1) * kStatChunk);
  double h = 0, m2 = 0, m4 = 0;
  for (int j = ch * kStatChunk + threadIdx.x; j < j1; j += 256) {
    double c = 0;
    for (int g = 0; g < L.Hkv; ++g) c += (double)pre[(size_t)g * L.T + j].x;
    const double p = c / Z;
    if (p > 0) h -= p * log(p);
    const double d = p - pbar, d2 = d * d;
    m2 += d2; m4 += d2 * d2;
  }
  h = block_sum_d(h, sm); m2 = block_sum_d(m2, sm); m4 = block_sum_d(m4, sm);
  if (threadIdx.x == 0) {
    double* o = mpart + ((size_t)b * nch + ch) * 3;
    st_dev_d(o, h); st_dev_d(o + 1, m2); st_dev_d(o + 2, m4);
    __builtin_amdgcn_s_waitcnt(0);                    // the partials are at the device's coherence point
    last = __hip_atomic_fetch_add(L.stat_ticket + b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nch - 1;
  }
  __syncthreads();
  if (!last) return;
  h = 0; m2 = 0; m4 = 0;
  for (int i = threadIdx.x; i < nch; i += 256) {
    const double* o = mpart + ((size_t)b * nch + i) * 3;
    h += ld_dev_d(o); m2 += ld_dev_d(o + 1); m4 += ld_dev_d(o + 2);
  }
  h = block_sum_d(h, sm); m2 = block_sum_d(m2, sm); m4 = block_sum_d(m4, sm);
  if (threadIdx.x != 0) return;
  __hip_atomic_store(L.stat_ticket + b, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
  m2 /= (double)n; m4 /= (double)n;
  L.stats[b * 3 + 0] = (float)h;
  L.stats[b * 3 + 1] = (float)m2;
  L.stats[b * 3 + 2] = m2 > 0 ? (float)(m4 / (m2 * m2)) : 0.f;
}

template <int D, int RT>
static hipError_t launch_prefill_t(const PrefillLaunch& a, float* rowc, hipStream_t s) {
  const int U = a.B * a.Hkv, MP = RT * 32;
  constexpr int NW = RT > 8 ? 8 : 4;
  const size_t shm = (size_t)MP * (2 * D + 16);
  if (shm + (size_t)MP * 8 > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_prefill_rows<D, RT, NW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_prefill_cols<D, RT, NW>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)(shm + (size_t)MP * 8));
    if (e != hipSuccess) return e;
  }
  dim3 grid(a.n_chunks, U);
  if (!a.have_rowc) {
    hipLaunchKernelGGL((k_prefill_rows<D, RT, NW>), grid, dim3(64 * NW), shm, s, a);
    hipLaunchKernelGGL(k_prefill_rowfinal, dim3(MP / 32, U), dim3(256), 0, s, a, MP, rowc);
  }
  const int nch = (a.T - a.W + kStatChunk - 1) / kStatChunk;
  double* zpart = reinterpret_cast<double*>(rowc + (size_t)U * MP);      // [U][n_chunks], then [B][nch][3]
  double* mpart = zpart + (size_t)U * a.n_chunks;
  hipLaunchKernelGGL((k_prefill_cols<D, RT, NW>), grid, dim3(64 * NW), shm + (size_t)MP * 8, s, a, (const float*)rowc, zpart);
  hipLaunchKernelGGL(k_prefill_stats, dim3(nch, a.B), dim3(256), 0, s, a, (const double*)zpart, mpart);
  return hipGetLastError();
}

// rowc: scratch [U][MP] floats followed by U*n_chunks + 3*B*ceil((T-W)/512) doubles for the statistics partials
hipError_t launch_prefill_stats(const PrefillLaunch& a, float* rowc, hipStream_t s) {
  const int M = a.G * a.W;
  int RT = 1;
  while (RT * 32 < M) RT *= 2;
  if (RT > 16) return hipErrorInvalidValue;
#define ARKV_PF(D_, RT_) if (a.D == D_ && RT == RT_) return launch_prefill_t<D_, RT_>(a, rowc, s);
  ARKV_PF(128, 1) ARKV_PF(128, 2) ARKV_PF(128, 4) ARKV_PF(128, 8) ARKV_PF(128, 16)
  ARKV_PF(64, 1) ARKV_PF(64, 2) ARKV_PF(64, 4) ARKV_PF(64, 8) ARKV_PF(64, 16)
#undef ARKV_PF
  return hipErrorInvalidValue;
}

}  // namespace arkv
