// Shared declarations of libarkv's host code and gfx950 kernels: data layout in HBM and launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace arkv {

constexpr int kGroup = 32;        // channels per (scale, zero) pair
constexpr int kMaxSplits = 128;   // split-K factor of the decode attention, upper bound
constexpr int kMaxLayersPerLaunch = 64;
constexpr int kMaxUnitsKnown = 64;     // launches with at most this many units can carry host-known token counts

// Cache memory of ALL layers.  Every array is [L*U][...] with U = B*H_kv units per layer, so that a
// launch over several layers is just a launch over more units.  "O pool": bf16 rows of Original
// tokens, slots [0, cnt.x) dense.  "Q pool": packed rows of Quantized tokens, slots [0, cnt.y) dense.
// A tailor compacts both pools in place; between tailors tokens are only appended to the O pool.
// Slots of per-step state (query, scale, final softmax constants) kept per unit: up to kRing-1 finished steps
// wait for their score update, one slot is written by the step in flight.
constexpr int kRing = 9;

// 32-bit metadata words of one packed K row
__host__ __device__ constexpr int metas_per_row(int D, int bits) { return bits == 8 ? 1 : D / kGroup; }
// tokens per block of the value rows' token-minor layout, and fp16 metadata words of one packed V row
constexpr int kVBlock = 32;
__host__ __device__ constexpr int vmeta_per_row(int D, int bits) { return bits == 8 ? 1 : 2 * (D / kGroup); }
// Where byte `col` of the value row in slot `slot` of a unit sits, relative to the unit's qvc (CB = bytes per
// row).  Within a block the bytes are ordered [8-token octet kb][lane n][column group i][token % 8], with
// n = col % NL, i = col / NL and NL = 16 lanes (8 for 2-bit rows, where lanes n and n + 8 read the same bytes): the 8
// tokens of ALL the columns a lane needs are contiguous, so a lane fetches them with 16-byte loads.
__host__ __device__ inline size_t vcode_index(int slot, int col, int CB, int bits) {
  const int NL = bits == 2 ? 8 : 16, NLD = CB / NL;
  const int t = slot % kVBlock;
  return ((((size_t)(slot / kVBlock) * 4 + t / 8) * NL + col % NL) * NLD + col / NL) * 8 + t % 8;
}
// Key codes of a row: the row's chunks (k-step kk, lane block blk) of CW = bits bytes (4 for 4-bit, 2 for 2-bit, 8
// for fp8 rows) are stored [blk][kk] instead of the canonical [kk][blk], so that everything lane block blk needs
// of a row is contiguous (one wide load per lane instead of one narrow load per k-step).  Canonical byte c -> stored.
__host__ __device__ inline int kcode_index(int c, int D, int bits) {
  const int KK = D / 32, CW = bits;
  const int kk = c / (4 * CW), blk = (c / CW) % 4;
  return (blk * KK + kk) * CW + c % CW;
}
// the same for fp16 metadata word m of the row (grouped formats: m = g for the scale, D/32 + g for the zero point)
__host__ __device__ inline size_t vmeta_index(int slot, int m, int MH) {
  return ((size_t)(slot / kVBlock) * MH + m) * kVBlock + slot % kVBlock;
}

struct Pools {
  int U;                // units per layer
  int capO, capQ;       // slots per unit: N and b
  int capQv;            // capQ rounded up to whole value blocks (kVBlock tokens): rows per unit of qvc / qvm
  int D, G, bits;
  // O pool
  uint16_t* ok;         // [LU][capO][D] bf16 keys
  uint16_t* ov;         // [LU][capO][D] bf16 values
  int32_t*  opos;       // [LU][capO] position of the token in the sequence
  float2*   oacc;       // [LU][capO] (s1, s2): running sums of attention and attention^2 (eq. 9)
  // Q pool
  uint8_t*  qkc;        // [LU][capQ][D*bits/8] key codes: canonical packing (bits = 8: one fp8 E4M3 byte per channel), bytes in
                        // the order of kcode_index
  uint32_t* qkm;        // [LU][capQ][metas_per_row] (fp16 scale | fp16 zero << 16) per group; bits = 8: one fp16 scale per row
  // Value rows are stored token-minor in blocks of kVBlock tokens, because PV contracts over tokens and a matrix-core
  // operand holds 8 consecutive contraction indices per lane: byte b of a token's canonical row (the same bytes as
  // in a canonical row: two 4-bit, four 2-bit or one fp8 code) sits at vcode_index within the unit's blocks.
  uint8_t*  qvc;        // [LU][capQv / kVBlock][D*bits/8 * kVBlock]
  // fp16 words: grouped formats [block][2][D/32][kVBlock] (scales of group g, then zero points of group g, one per
  // token); fp8 rows [block][kVBlock] (the row scales)
  uint16_t* qvm;        // [LU][capQv / kVBlock][vmeta_per_row][kVBlock]
  int32_t*  qpos;       // [LU][capQ]
  float2*   qacc;       // [LU][capQ]
  // per unit
  int2*     cnt;        // [LU] (tokens in O pool, tokens in Q pool)
  float2*   fin;        // [kRing][LU][G] (row max in base-2 units, 1/denominator) of the latest steps, ring by step
  size_t    fin_stride; // LU*G
  uint16_t* qprev;      // [kRing][LU][G][D] bf16 queries of the latest steps (the score update recomputes logits)
  float*    qscale;     // [kRing][LU] softmax scale * log2(e) those queries were used with
  float*    part;       // [LU][max_splits][G][D+2] split-K partials: acc[D], max, sum
  int       max_splits;
  int*      ticket;     // [LU] splits of the unit finished in the current launch (0 between launches)
  float*    outf;       // [LU][G][D] fp32 output of the latest step (parity hook)
  int32_t*  n_o;        // [LU] Original target of the unit's layer/sequence
  int32_t*  nb;         // [LU] survivors outside the window (n_o + n_q) of the unit's layer/sequence
  // tailor scratch
  uint64_t* keys;       // [LU][capO+capQ] selection keys of the latest tailor (0 = not eligible)
  uint64_t* thr;        // [LU][2] keys of rank n_o and rank b
  int32_t*  plan;       // [LU][kPlanHdr + 2*capO + 3*capQ... ] see arkv_tailor.hip
  int       plan_stride;
};

constexpr int kPlanHdr = 16;
// plan header fields (int32 each)
enum { PL_CO_NEW = 0, PL_CQ_NEW, PL_N_DEM, PL_N_QMOV, PL_N_OMOV, PL_N_ELIG, PL_CO_OLD, PL_CQ_OLD };

// Reciprocals for the decode kernel's split cut points (see split_range)
struct SplitRecip { unsigned inv_s, inv_wq; };          // ceil(2^32 / S), ceil(2^32 / wq) (unused when S or wq is 1)
__host__ __device__ inline SplitRecip split_recip(int S, int wq) {
  SplitRecip r;
  r.inv_s = S > 1 ? (unsigned)(0xFFFFFFFFull / (unsigned)S) + 1u : 0u;
  r.inv_wq = wq > 1 ? (unsigned)(0xFFFFFFFFull / (unsigned)wq) + 1u : 0u;
  return r;
}

struct DecodeLaunch {
  const uint16_t* q;      // [n][B][Hq][D]
  const uint16_t* k_new;  // [n][B][Hkv][D]
  const uint16_t* v_new;
  uint16_t* out;          // [n][B][Hq][D]
  int unit_begin;         // first global unit (= layer_begin * U)
  int n_units;            // n * U
  int units_per_layer;
  int splits;
  int position;           // P of the token being appended
  int n_pending;          // steps whose probabilities are not yet added to (s1,s2), 0..kRing-1; the j-th oldest
                          // of them used ring slot (slot - n_pending + j) mod kRing
  int slot;               // ring slot of fin/qprev/qscale this step writes
  int fold;               // 1: this launch adds the pending steps to (s1,s2)
  int wq;                 // cost of a packed row in sixteenths of a bf16 row (split balancing)
  unsigned inv_splits, inv_wq;   // ceil(2^32 / splits), ceil(2^32 / wq): the split cut points without divisions
  int part_unit0;         // global unit whose partials and ticket come first in Pools::part / ticket (0: arrays of the
                          // whole cache; unit_begin: a buffer that holds this launch only)
  int cnt_known;          // 1: cnt_o / cnt_q below are the units' token counts (saves a dependent load)
  int cnt_o[kMaxUnitsKnown], cnt_q[kMaxUnitsKnown];
  float scale2[kMaxLayersPerLaunch];  // softmax scale * log2(e), per launched layer
};

struct TailorLaunch {
  int unit_begin, n_units;
  int position;       // P of the latest token
  int t_prefill;      // T
  int window;
  float gamma;
  int n_pending, slot;  // pending steps to add to (s1,s2) before ranking; slot the NEXT step would write
};

struct CommitLaunch {
  const uint16_t* k;  // [B][Hkv][T][D]
  const uint16_t* v;
  const float2* pre;  // [U][T] window sums (s1, s2) from the prefill scorer
  int unit_begin, n_units;
  int T, window;
  float gamma;
  int select;         // 1: T >= N, run the first tailor; 0: copy everything as Original
};

struct PrefillLaunch {
  const uint16_t* q_win;  // window query rows: row i of head h at q_win + h * q_head_stride + i * D
  const uint16_t* k;      // [B][Hkv][T][D]
  float2* pre;            // [U][T]  out: (s1, s2)
  float2* rowstat;        // [U][chunks][G*W] (row max base-2, row sum) partials
  float* stats;           // [B][3]
  int* stat_ticket;       // [B] workgroups of the sequence's statistics kernel that finished (0 between calls)
  int B, Hkv, G, W, D, T;
  size_t q_head_stride;   // elements between heads (W*D for a packed [B][Hq][W][D] tensor)
  int have_rowc;          // 1: the row constants are already in the scratch (attention pass), skip the first pass
  const float* lse;       // not null: the caller's log-sum-exp [U][G][W] (natural log), from which the column pass
                          // takes its row constants itself (have_rowc is 1 then, and the scratch rows are not read)
  int chunk;              // keys per workgroup
  int n_chunks;
  float scale2;
};

hipError_t launch_decode(const Pools& P, const DecodeLaunch& a, hipStream_t s, hipEvent_t ev0 = nullptr,
                         hipEvent_t ev1 = nullptr);  // ev0/ev1: recorded around the attention kernel
// Split-K scratch in static device memory (for the entry point that must not allocate): one array per GPU.
constexpr size_t kStaticScratchBytes = 4u << 20;   // tickets of up to kStaticUnits units, then partials
constexpr int kStaticUnits = 4096;
hipError_t static_scratch_setup();                  // once per device, with that device current (synchronous)
hipError_t static_scratch_get(float** part, int** ticket, size_t* part_floats);   // pointers for the current device
// Profiling builds only (built = false otherwise): in-kernel timestamps of the latest launches.
hipError_t phase_trace_decode(int which, unsigned long long* host, int n_wg, bool* built);
hipError_t phase_trace_attn(unsigned long long* host, bool* built);
hipError_t launch_flush_scores(const Pools& P, int unit_begin, int n_units, int n_pending, int slot, hipStream_t s);
hipError_t launch_tailor(const Pools& P, const TailorLaunch& a, hipStream_t s);
hipError_t launch_commit(const Pools& P, const CommitLaunch& a, uint64_t* commit_keys /*[U][T]*/, hipStream_t s);
// n_o_seq, nb_seq: HOST [batch]; written to the units of one layer (unit_begin = layer * U) on the stream
hipError_t launch_set_budgets(const Pools& P, int unit_begin, int hkv, int batch, const int32_t* n_o_seq,
                              const int32_t* nb_seq, hipStream_t s);
// Causal prefill attention of T_q queries (positions [T - T_q, T)) over T keys.
struct AttnLaunch {
  const uint16_t* q;      // [B][Hq][Tq][D]
  const uint16_t* k;      // [B][Hkv][T][D]
  const uint16_t* v;
  uint16_t* out;          // [B][Hq][Tq][D]
  float* outf;            // [B][Hq][Tq][D] the same output before its rounding to bf16 (parity hook), or null
  float* rowc;            // [U][MP] max + log2(sum) of the last W rows per head, or null
  int B, Hq, Hkv, D, T, Tq, W, MP;
  float scale2;
};
hipError_t launch_prefill_attn(const AttnLaunch& a, hipStream_t s);
hipError_t launch_prefill_stats(const PrefillLaunch& a, float* rowc /*[U][MP] scratch*/, hipStream_t s);

}  // namespace arkv
