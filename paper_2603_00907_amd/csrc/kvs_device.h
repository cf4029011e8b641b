// Internal declarations shared by the host layer and the gfx950 kernels of libkvs.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvs.h"
#include "kvs_debug.h"

namespace kvs {

// Current value of a testing switch (kvs_debug.h): one relaxed atomic load, no environment lookup.
int debug_switch(kvs_debug_switch which);

// Units of one launch ("group").  Up to kInlineUnits unit descriptors travel by value in the kernel arguments; a
// larger group (many short units: the streaming regime's caches of 2.5 K rows) has its descriptors written to the
// workspace first, by small kernels that carry them in THEIR arguments, kInlineUnits at a time.  A group takes
// kInlineUnits units whatever their lengths, and more as long as it has fewer than kGroupTokens tokens (64 units of
// 32 K tokens: longer launches gain nothing), up to kMaxGroupUnits units.
constexpr int kInlineUnits = 64;
constexpr int kMaxGroupUnits = 1024;
#ifndef KVS_GROUP_TOKENS
#define KVS_GROUP_TOKENS (64ll * 32768)
#endif
constexpr long long kGroupTokens = KVS_GROUP_TOKENS;
constexpr int kMaxChunks = 64;           // token chunks (= score workgroups) per unit
constexpr int kMinChunkLen = 256;        // tokens
constexpr int kMaxChunkLen = 2048;       // tokens
constexpr int kScoreWorkgroups = 1024;   // score workgroups a launch aims for (4 per CU)
constexpr int kObarMinChunk = 1024;      // tokens per workgroup of the o_bar pass (at most kMaxChunks per unit)
#ifndef KVS_MERGE_TOKENS
#define KVS_MERGE_TOKENS 256
#endif
constexpr int kMergeTokens = KVS_MERGE_TOKENS;   // tokens per merge workgroup
constexpr int kWave = 64;
// K plus V bytes of one launch above which rows are streamed past the caches (256 MB of memory-side
// cache: below that, a sweep finds the rows its predecessor left there)
constexpr long long kStreamBytes = 192ll << 20;
// One-pass score kernel: bytes of K (bf16 rows) that one of its work items keeps in LDS between the statistics
// phase and the alpha_bar phase (one workgroup per CU: 128 KB of K + 16 KB of Q + tables of 160 KB)
constexpr int kFusedChunkBytes = 128 * 1024;

// One (sequence, KV head).  Rows are in elements of D, not bytes.
struct Unit {
  long long in_row;     // first row in K, V, alpha_bar, edge_mask, slot_of_token
  long long out_row;    // first row in K_out, V_out, counts_out
  int len;              // cached tokens
  int n_out;            // output rows: min(len, budget)
  int chunk_len;        // tokens per score chunk (multiple of 64)
  int n_chunks;         // ceil(len / chunk_len), <= kMaxChunks
  int chunk_base;       // chunks of the launch's earlier units
  int m_base;           // merge workgroups (kMergeTokens tokens each) of the launch's earlier units
  int index;            // position of the unit in the caller's problem (indexes Q, o_bar, partials)
  int o_base;           // o_bar-pass workgroups of the launch's earlier units
  int f_base;           // work items of the one-pass score kernel that belong to the launch's earlier units
  int s_base;           // select workgroups of the launch's earlier units (a unit has one, or several parts)
};

// Work items of the one-pass score kernel: chunks of kFusedChunkBytes of K rows (a function of D and the length).
__host__ __device__ inline int fused_chunk_len(int D) { return kFusedChunkBytes / (D * 2); }
__host__ __device__ inline int fused_chunks(int len, int D) {
  const int cl = fused_chunk_len(D);
  return (len + cl - 1) / cl;
}

// Chunking of the o_bar pass over V: a function of the unit's length only.
__host__ __device__ inline int obar_chunk_len(int len) {
  const int per = (len + kMaxChunks - 1) / kMaxChunks;
  const int rounded = (per + kWave - 1) / kWave * kWave;
  return rounded > kObarMinChunk ? rounded : kObarMinChunk;
}
__host__ __device__ inline int obar_chunks(int len) {
  const int cl = obar_chunk_len(len);
  return (len + cl - 1) / cl;
}

// Selection over several workgroups ("parts") per unit.  A part keeps at most kSelPartKeys edge scores in LDS; what
// the parts of a unit exchange goes through kSelSharedInts unsigned ints of device memory per unit of the launch,
// which must be zero when the select kernel starts (the score finalize kernel of the same call clears them):
//   [kSelNotMin] ~(smallest key), [kSelMax] largest key, [kSelNCand] candidates listed so far,
//   [kSelArrive + phase] parts that finished a phase (bit kSelGaveUp: a part ran out of time there),
//   [kSelPartLow + part] keys of a part in the bins below the threshold's,
//   [kSelHist + bin] histogram of the first digit, [kSelCand + i] keys of the threshold's bin and
//   [kSelCandPart + i] the parts they came from.
constexpr int kSelUnitKeys = 32768;       // keys that ONE workgroup can keep in LDS (the full-size select kernel)
constexpr int kSelMaxParts = 32;
constexpr int kSelPartKeys = 8192;
constexpr int kSelMinPartKeys = 2048;     // parts are not made smaller than this unless a test asks for it
constexpr int kSelNotMin = 0, kSelMax = 1, kSelNCand = 2, kSelArrive = 4, kSelPhases = 3;
constexpr unsigned int kSelGaveUp = 1u << 16;
constexpr int kSelPartLow = 16;
constexpr int kSelHist = 64, kSelHistBins = 2048;
constexpr int kSelCand = kSelHist + kSelHistBins, kSelCandMax = 2048;
constexpr int kSelCandPart = kSelCand + kSelCandMax;
constexpr int kSelSharedInts = kSelCandPart + kSelCandMax;
static_assert(kSelPartLow + kSelMaxParts <= kSelHist && kSelSharedInts % 4 == 0, "layout of the exchange area");

struct UnitTable {
  const Unit* ext;      // DEVICE: the descriptors of a group of more than kInlineUnits units, else null
                        // (first, beside n_units: a kernel's first scalar load then brings both)
  int n_units;
  int total_chunks;
  int total_mblocks;
  int total_ochunks;
  int total_fitems;     // work items of the one-pass score kernel
  int total_sparts;     // select workgroups
  const Unit* host;     // HOST: the same descriptors for the launchers (meaningless on the device), else null
  Unit u[kInlineUnits]; // the descriptors of a smaller group

  // Descriptor i, on either side.  On the device the external table is read through the constant address space:
  // the index is wavefront-uniform, so these are scalar loads like those of the kernel arguments.
  __host__ __device__ __forceinline__ Unit unit(int i) const {
#if defined(__HIP_DEVICE_COMPILE__)
    if (ext != nullptr) return ((const __attribute__((address_space(4))) Unit*)ext)[i];
    return u[i];
#else
    return host != nullptr ? host[i] : u[i];
#endif
  }
};

struct Shape {
  int R;            // query rows per unit (G*W)
  int D;            // head dim
  int n_sink;
  int n_recent;
  float scale_log2; // logit scale * log2(e): logits are kept in the base-2 domain
  int stream;       // 1: the launch's K and V exceed the last-level cache, rows are read non-temporally
  int rule;         // kvs_key_rule of the merged Key
  int causal;       // 0, or the window W when query row q only sees the rows up to its own position n - W + q % W
  int dec_chunk;    // decode attention: rows per workgroup, at least (chosen per launch, see launch_decode)
  int o_from_score; // where the partial sums of o_bar are: 0: o_part, one per chunk of the o_bar pass; 1: o_part, one
                    // per SCORE chunk (written by sweep 1); 2: fo_part, one per work item of the one-pass score kernel
};

// How many partials of o_bar a unit has, and where its partial c starts (index of its first float).
__host__ __device__ inline int obar_partials(const Shape& sh, const Unit& un) {
  return sh.o_from_score == 2 ? fused_chunks(un.len, sh.D) : sh.o_from_score == 1 ? un.n_chunks : obar_chunks(un.len);
}
__host__ __device__ inline size_t obar_partial_at(const Shape& sh, const Unit& un, int c) {
  return sh.o_from_score == 2 ? ((size_t)un.f_base + c) * sh.D : ((size_t)un.index * kMaxChunks + c) * sh.D;
}

// Workspace carve-up (all offsets multiples of 256 bytes).
struct Workspace {
  float2* stats_part;   // [n_units][kMaxChunks][R]  (running max, sum) of every chunk, base-2 domain
  float* c_row;         // [n_units][R]  unit-wide normaliser of every query row, see score_finalize_kernel
  float* o_part;        // [n_units][kMaxChunks][D]  partial o_bar of every chunk of the o_bar pass
  float* alpha_bar;     // [rows]    (kvs_step only)
  float* o_bar;         // [n_units][D] (kvs_step only)
  uint8_t* edge_mask;   // [rows]    (kvs_step only, when the caller keeps it internal)
  int32_t* slot;        // [rows]
  // one-pass score kernel (bf16, 65..128 query rows); sized for the largest launch group, null otherwise
  float* fstats;        // [work items][R]  log2 of the sum of 2^logit over the item's tokens, for every query row
  float* fo_part;       // [work items][D]  partial o_bar of every item
  unsigned int* fsync;  // kFusedSyncInts counters and flags, then one entry per work item (items given up on)
  unsigned int* sel_shared;  // [kInlineUnits][kSelSharedInts]  exchange area of the split selection (only groups of
                             // at most kInlineUnits units spread a unit's selection over workgroups)
  Unit* unit_tab;            // [kMaxGroupUnits]  descriptors of a group of more than kInlineUnits units
  size_t bytes;
};

// Layout of Workspace::fsync (unsigned ints).
constexpr int kFusedTicket = 0;                       // next work item
constexpr int kFusedDeferred = 32;                    // number of items handed to the second kernel
constexpr int kFusedDone = 64;                        // [kInlineUnits] items of the unit whose statistics are out
constexpr int kFusedSyncInts = 64 + kInlineUnits;     // the list of deferred items starts here
                                                      // (the one-pass kernel's groups have at most kInlineUnits units)
// A normaliser c_row[unit][q] that the one-pass kernel has not produced yet holds this bit pattern (a NaN that no
// arithmetic yields): the kernel's workgroups poll the words themselves, so no separate flag has to travel.
constexpr unsigned int kFusedNotYet = 0xffffffffu;

// Device helpers --------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// float -> bf16 bits, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return f32_to_bf16(lo) | (f32_to_bf16(hi) << 16);
}

// 16-byte row piece -> floats.  T = float: 4 values; T = bf16 (uint16_t): 8 values.
template <typename T> struct Piece;
template <> struct Piece<float> {
  static constexpr int N = 4;
  __device__ __forceinline__ static void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ __forceinline__ static uint4 pack(const float* f) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
};
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// two floats -> packed bf16 pair with the hardware converter (v_cvt_pk_bf16_f32, round to nearest even)
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  const f32x2_t f = {lo, hi};
  const bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return *reinterpret_cast<const uint32_t*>(&b);
}

template <> struct Piece<uint16_t> {
  static constexpr int N = 8;
  __device__ __forceinline__ static void unpack(const uint4& r, float* f) {
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
  }
  __device__ __forceinline__ static uint4 pack(const float* f) {
    return make_uint4(cvt_pk_bf16(f[0], f[1]), cvt_pk_bf16(f[2], f[3]), cvt_pk_bf16(f[4], f[5]), cvt_pk_bf16(f[6], f[7]));
  }
};

// Sum over the LPR (8, 16 or 32) adjacent lanes that share a row; every lane gets the total.
// gfx950 has no xor-by-4/8 DPP pattern, but once the four lanes of a quad agree, mirroring a
// half-row and then a row swaps exactly the partners a butterfly would.
template <int LPR>
__device__ __forceinline__ float row_group_sum(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // row_half_mirror
  if (LPR >= 16)
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));  // row_mirror
  if (LPR >= 32) x += __shfl_xor(x, 16, kWave);
  return x;
}

// Causal window: the last row that query row `qrow` of a unit with n rows attends to.
__device__ __forceinline__ int last_seen_row(int causal_w, int n, int qrow) {
  return causal_w > 0 ? n - causal_w + qrow % causal_w : 0x7fffffff;
}

// The unit's normalisers c[q] (written by the finalize kernel between the two sweeps) -> LDS.
__device__ __forceinline__ void load_row_consts(const float* __restrict__ c_row, int unit_index, int R, float* sm_c) {
  for (int q = threadIdx.x; q < R; q += blockDim.x) sm_c[q] = c_row[(size_t)unit_index * R + q];
  __syncthreads();
}

// The last unit whose running count BASE (chunks, merge workgroups, ... of the launch's earlier units) is at most x:
// the unit that work item x of the launch belongs to.  A binary search, because the table lives in the kernel
// arguments and every probe is a scalar load that the next one depends on (about a quarter of a microsecond when
// it misses the scalar cache: walking the table unit by unit cost a 64-unit select launch 15 of its 37 us).
template <int Unit::*BASE>
__device__ __forceinline__ int find_unit_by(const UnitTable& tab, int x) {
  int lo = 0, hi = tab.n_units - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (tab.unit(mid).*BASE <= x) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}
// Which unit a workgroup of a chunk-indexed launch works on.
__device__ __forceinline__ int find_unit(const UnitTable& tab, int chunk) {
  return find_unit_by<&Unit::chunk_base>(tab, chunk);
}

// Launchers (defined next to their kernels).  All enqueue on `stream` and return the launch status.
// The descriptors of a group of more than kInlineUnits units (host memory) into the workspace, by kernels that
// carry them in their arguments.
hipError_t launch_unit_table(const Unit* units, int n_units, Unit* dst, hipStream_t stream);
// Unit-wide softmax statistics from the chunks' partial ones (one small workgroup per unit).
// (it also zeroes ws.sel_shared for the selection that follows, when there is one)
hipError_t launch_score_finalize(const UnitTable& tab, const Shape& sh, const Workspace& ws, hipStream_t stream);
// Both score sweeps: chunk statistics, the finalize kernel, then alpha_bar.
// counts_in (here and below): cardinalities of the input rows when the cache is already a merged one, or null.
// V non-null: the caller also needs o_bar; where the score kernel can carry the pass over V along, it does,
// leaves the partial sums in the workspace and sets *o_layout to where they are (a value for Shape::o_from_score
// other than 0: the caller then skips the separate pass and tells the consumers).
hipError_t launch_score(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* Q, const void* K,
                        const int32_t* counts_in, float* alpha_bar, const Workspace& ws, hipStream_t stream,
                        const void* V = nullptr, int* o_layout = nullptr);
// One launch, several kinds of workgroups: the first `with_select ? tab.total_sparts : 0` select edges (one workgroup
// per unit, or several parts per unit that meet through sel_shared), the others stream one chunk of V each into
// o_part (skipped when V is null).
// A third kind (o_bar_out non-null, one workgroup per unit) adds up the partial sums that a score kernel left
// (sh.o_from_score says where) into o_bar_out[unit][D].
// sel_shared: the zeroed exchange area (see kSelSharedInts), needed when any unit has more than one part.
hipError_t launch_select_obar(const UnitTable& tab, const Shape& sh, kvs_dtype dt, bool with_select,
                              const float* alpha_bar, uint8_t* edge_mask, int32_t* slot, const void* V,
                              const int32_t* counts_in, float* o_part, hipStream_t stream,
                              const float* parts_in = nullptr, float* o_bar_out = nullptr,
                              unsigned int* sel_shared = nullptr);
// Zeroes the exchange area of the launch's units (callers that did not run the score kernels before the selection).
hipError_t launch_select_clear(const UnitTable& tab, unsigned int* sel_shared, hipStream_t stream);
// How many select workgroups a unit gets in a launch of n_units units on a chip of n_cus compute units
// (mode: the KVS_DEBUG_SELECT_SPLIT switch).  1: the single-workgroup selection.
int select_parts(const Unit& un, const Shape& sh, int n_units, int n_cus, int mode);
// o_bar[u] = sum of the unit's partial sums, in chunk order (only when o_bar itself is an output).
hipError_t launch_obar_reduce(const UnitTable& tab, const Shape& sh, const float* parts, float* o_bar,
                              hipStream_t stream);
// One-pass score for bf16 windows of 65..128 rows (kvs_score_fused.hip): K is read once and kept in LDS between
// the statistics and the alpha_bar phase; the pass over V rides along (partials in ws.fo_part).
bool score_fused_supported(const UnitTable& tab, const Shape& sh, kvs_dtype dt);
hipError_t launch_score_fused(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                              const int32_t* counts_in, float* alpha_bar, const Workspace& ws, hipStream_t stream);
// Exactly one of o_bar (final values) and o_part (chunk sums, added up by every workgroup) is non-null.
hipError_t launch_merge(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* K, const void* V,
                        const int32_t* counts_in, const float* alpha_bar, const float* o_bar, const float* o_part,
                        const uint8_t* edge_mask,
                        const int32_t* slot, void* K_out, void* V_out, int32_t* counts, hipStream_t stream);

// The same pass with A_t and C_t read from arrays instead of formed from alpha_bar and o_bar (per-query aggregation).
hipError_t launch_merge_norms(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* K, const void* V,
                              const int32_t* counts_in, const float* a_tok, const float* c_edge,
                              const uint8_t* edge_mask, const int32_t* slot, void* K_out, void* V_out, int32_t* counts,
                              hipStream_t stream);
// Per-query aggregation (bf16, every unit at least 32 rows): a_tok, c_edge from Q, K, V and the rows' normalisers
// c_row that the score sweeps leave.  o_part: [chunks of the launch][R][D] fp32; o_hi, o_lo: [n_units][R][D] bf16;
// oo: [n_units][R].
hipError_t launch_per_query_norms(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                                  const int32_t* counts_in, const float* c_row, float* o_part, uint16_t* o_hi,
                                  uint16_t* o_lo, float* oo, float* a_tok, float* c_edge, hipStream_t stream);
// The same for fp32 inputs (any unit length, vector ALU).  o: [n_units][R][D] fp32.
hipError_t launch_per_query_norms_f32(const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                                      const void* V, const int32_t* counts_in, const float* c_row, float* o_part,
                                      float* o, float* a_tok, float* c_edge, hipStream_t stream);

// Decode attention over a (merged) cache: chunk partials into `part`, then out[n_units, R, D].
hipError_t launch_decode(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* Q, const void* K,
                         const void* V, const int32_t* counts, float* part, float* out, hipStream_t stream);

}  // namespace kvs
