// Host layer of libkvs: argument validation, workspace carve-up, unit tables, launch sequencing.
// Everything that can fail because of the arguments fails here, before the first launch.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "kvs_device.h"

namespace kvs {

hipError_t launch_score_valu(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* Q, const void* K,
                             const int32_t* counts_in, float* alpha_bar, const Workspace& ws, hipStream_t stream);
hipError_t launch_score_mfma(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* Q, const void* K,
                             const int32_t* counts_in, float* alpha_bar, const Workspace& ws, const void* V,
                             hipStream_t stream);
bool score_mfma_supported(const UnitTable& tab, const Shape& sh, kvs_dtype dt);
bool score_mfma_takes_values(const Shape& sh, kvs_dtype dt);

// ---- testing switches (kvs_debug.h): process-global, initial values read from the environment once, at load
namespace {
std::atomic<int> g_switch[KVS_DEBUG_N_SWITCHES];

int env_choice(const char* name, const char* one, const char* two) {
  const char* e = std::getenv(name);
  if (e == nullptr) return 0;
  if (one && std::strcmp(e, one) == 0) return 1;
  if (two && std::strcmp(e, two) == 0) return 2;
  return 0;
}

struct SwitchInit {
  SwitchInit() {
    g_switch[KVS_DEBUG_SCORE_PATH] = env_choice("KVS_SCORE_PATH", "valu", nullptr);
    g_switch[KVS_DEBUG_SCORE_WIDE] = env_choice("KVS_SCORE_WIDE", "0", nullptr);
    g_switch[KVS_DEBUG_FUSE_OBAR] = env_choice("KVS_FUSE_OBAR", "0", "1");
    g_switch[KVS_DEBUG_DECODE_PATH] = env_choice("KVS_DECODE_PATH", "valu", "mfma");
    const char* c = std::getenv("KVS_SCORE_CHUNK");
    g_switch[KVS_DEBUG_SCORE_CHUNK] = c ? std::max(0, std::atoi(c)) : 0;
    g_switch[KVS_DEBUG_VERBOSE] = std::getenv("KVS_VERBOSE") != nullptr;
    g_switch[KVS_DEBUG_SCORE_FUSED] = env_choice("KVS_SCORE_FUSED", nullptr, "1");
    const char* sp = std::getenv("KVS_SELECT_SPLIT");
    g_switch[KVS_DEBUG_SELECT_SPLIT] = sp ? std::min(3, std::max(0, std::atoi(sp))) : 0;
    const char* t = std::getenv("KVS_FUSED_WAIT_US");
    g_switch[KVS_DEBUG_FUSED_WAIT_US] = t ? std::max(0, std::atoi(t)) + 1 : 0;
    const char* g = std::getenv("KVS_FUSED_STAGGER");
    g_switch[KVS_DEBUG_FUSED_STAGGER] = g ? std::max(0, std::atoi(g)) + 1 : 0;
    const char* gu = std::getenv("KVS_GROUP_UNITS");
    g_switch[KVS_DEBUG_GROUP_UNITS] = gu ? std::max(0, std::atoi(gu)) : 0;
  }
} g_switch_init;
}  // namespace

int debug_switch(kvs_debug_switch which) { return g_switch[which].load(std::memory_order_relaxed); }

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Plan {
  int n_units = 0;
  Shape shape{};
  kvs_dtype dtype = KVS_F32;
  size_t elt = 4;
  long long rows_in = 0, rows_out = 0;
  long long fused_items = 0;     // work items of the largest launch group when the one-pass score kernel applies
  std::vector<Unit> units;       // chunk_base / m_base filled per launch group
  int group_cap = kInlineUnits;  // most units of a launch group
  Unit* dev_table = nullptr;     // where a group of more than kInlineUnits units keeps its descriptors (workspace), or
                                 // null: the call has no such memory and its groups stay within kInlineUnits
  hipStream_t stream = nullptr;  // the call's stream (the descriptors are written on it)
};

// One past the last unit of the launch group that starts at unit `first`.
int group_end(const Plan& plan, int first, int cap) {
  long long tokens = 0;
  int i = first;
  while (i < plan.n_units && i - first < cap && (i - first < kInlineUnits || tokens < kGroupTokens)) {
    tokens += plan.units[i++].len;
  }
  return i;
}

kvs_status make_plan(const kvs_problem* p, Plan* plan) {
  if (p == nullptr) return KVS_ERR_INVALID_ARG;
  if (p->n_units < 1 || p->group < 1 || p->window < 1) return KVS_ERR_INVALID_ARG;
  if ((long long)p->group * p->window > KVS_MAX_Q_ROWS) return KVS_ERR_INVALID_ARG;
  if (p->head_dim != 64 && p->head_dim != 128) return KVS_ERR_INVALID_ARG;
  if (p->n_sink < 0 || p->n_recent < 0) return KVS_ERR_INVALID_ARG;
  // (a caller may have put any integer into the enum fields: they are read as the ints they are in C)
  int io_dtype, key_rule;
  std::memcpy(&io_dtype, &p->io_dtype, sizeof(int));
  std::memcpy(&key_rule, &p->key_rule, sizeof(int));
  static_assert(sizeof(p->io_dtype) == sizeof(int) && sizeof(p->key_rule) == sizeof(int), "C enums");
  if (io_dtype != KVS_F32 && io_dtype != KVS_BF16) return KVS_ERR_DTYPE;
  if (!(p->scale >= 0.f) || !std::isfinite(p->scale)) return KVS_ERR_INVALID_ARG;
  if (!p->len || !p->budget || !p->in_row || !p->out_row) return KVS_ERR_INVALID_ARG;
  if (key_rule != KVS_RULE_HESSIAN && key_rule != KVS_RULE_DIAGONAL && key_rule != KVS_RULE_MEAN) {
    return KVS_ERR_INVALID_ARG;
  }

  plan->n_units = p->n_units;
  plan->dtype = p->io_dtype;
  plan->elt = (p->io_dtype == KVS_F32) ? 4 : 2;
  plan->shape.R = p->group * p->window;
  plan->shape.D = p->head_dim;
  plan->shape.n_sink = p->n_sink;
  plan->shape.n_recent = p->n_recent;
  plan->shape.rule = (int)p->key_rule;
  if (p->causal != 0 && p->causal != 1) return KVS_ERR_INVALID_ARG;
  plan->shape.causal = p->causal ? p->window : 0;
  const double scale = (p->scale == 0.f) ? 1.0 / std::sqrt((double)p->head_dim) : (double)p->scale;
  plan->shape.scale_log2 = (float)(scale * 1.4426950408889634);
  plan->units.resize(p->n_units);

  for (int u = 0; u < p->n_units; ++u) {
    const long long len = p->len[u], budget = p->budget[u];
    // (kernels address a unit's rows with 32-bit byte offsets: KVS_MAX_LEN rows of 512 bytes stay below 4 GB)
    if (len < 1 || len > KVS_MAX_LEN || p->in_row[u] < 0 || p->out_row[u] < 0) return KVS_ERR_INVALID_ARG;
    if (p->causal && len < p->window) return KVS_ERR_INVALID_ARG;   // the window's own rows are part of the cache
    if (budget < 1) return KVS_ERR_BUDGET;
    if (len > budget && budget < (long long)p->n_sink + 1 + p->n_recent) return KVS_ERR_BUDGET;
    Unit& un = plan->units[u];
    un.in_row = p->in_row[u];
    un.out_row = p->out_row[u];
    un.len = (int)len;
    un.n_out = (int)std::min(len, budget);
    un.chunk_len = 0;                 // set below, once the total amount of work is known
    un.n_chunks = 0;
    un.chunk_base = un.m_base = 0;
    un.index = u;
    un.o_base = 0;
    un.f_base = 0;
    un.s_base = 0;
    plan->rows_in = std::max(plan->rows_in, un.in_row + len);
    plan->rows_out = std::max(plan->rows_out, un.out_row + (long long)un.n_out);
  }
  // Score chunks (one workgroup each): long enough that a workgroup's prologue (Q block, statistics)
  // is a small part of its life, short enough that one launch (the first group of units) still
  // has a few workgroups for every slot of the chip; never more than kMaxChunks per unit.
  // (the one-pass score kernel keeps per-unit counters for kInlineUnits units; a test may ask for smaller groups)
  plan->group_cap = debug_switch(KVS_DEBUG_SCORE_FUSED) ? kInlineUnits : kMaxGroupUnits;
  if (const int forced = debug_switch(KVS_DEBUG_GROUP_UNITS)) plan->group_cap = std::min(forced, kMaxGroupUnits);
  {
    long long total = 0;
    for (int u = 0; u < group_end(*plan, 0, plan->group_cap); ++u) total += p->len[u];
    // (a launch of up to a million tokens gets half as many workgroups, one round of two per CU: the streaming
    // workload's 256 caches of 2560 rows take 0.265 ms per step that way against 0.273)
    long long want = total / (total <= (1ll << 20) ? kScoreWorkgroups / 2 : kScoreWorkgroups);
    if (const int forced = debug_switch(KVS_DEBUG_SCORE_CHUNK)) want = forced;   // tuning aid
    want = std::min<long long>(std::max<long long>(want, kMinChunkLen), kMaxChunkLen);
    for (int u = 0; u < p->n_units; ++u) {
      Unit& un = plan->units[u];
      const long long per = std::max<long long>(want, (un.len + kMaxChunks - 1) / kMaxChunks);
      un.chunk_len = (int)((per + kWave - 1) / kWave * kWave);
      un.n_chunks = (un.len + un.chunk_len - 1) / un.chunk_len;
    }
  }
  // the one-pass score kernel (bf16, 65..128 query rows, every unit at least a tile long) keeps per-item tables
  if (plan->dtype == KVS_BF16 && plan->shape.R > 64 && plan->shape.R <= 128) {
    const int cap = std::min(plan->group_cap, kInlineUnits);
    for (int first = 0, end; first < p->n_units; first = end) {
      end = group_end(*plan, first, cap);
      long long items = 0;
      for (int u = first; u < end; ++u) items += fused_chunks(plan->units[u].len, plan->shape.D);
      plan->fused_items = std::max(plan->fused_items, items);
    }
  }
  // the units' row ranges must not overlap, on the input and on the output side
  std::vector<std::pair<long long, long long>> in(p->n_units), out(p->n_units);
  for (int u = 0; u < p->n_units; ++u) {
    in[u] = {plan->units[u].in_row, plan->units[u].in_row + plan->units[u].len};
    out[u] = {plan->units[u].out_row, plan->units[u].out_row + plan->units[u].n_out};
  }
  std::sort(in.begin(), in.end());
  std::sort(out.begin(), out.end());
  for (int u = 1; u < p->n_units; ++u) {
    if (in[u].first < in[u - 1].second || out[u].first < out[u - 1].second) return KVS_ERR_INVALID_ARG;
  }
  return KVS_OK;
}

// Workspace layout.  `base` may be null (sizing only).
Workspace carve(const Plan& plan, void* base) {
  Workspace w{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* ptr = base ? (char*)base + off : nullptr;
    off += align_up(bytes);
    return (void*)ptr;
  };
  const size_t nu = (size_t)plan.n_units;
  w.stats_part = (float2*)take(nu * kMaxChunks * plan.shape.R * sizeof(float2));
  w.c_row = (float*)take(nu * plan.shape.R * sizeof(float));
  w.o_part = (float*)take(nu * kMaxChunks * plan.shape.D * sizeof(float));
  w.alpha_bar = (float*)take((size_t)plan.rows_in * sizeof(float));
  w.o_bar = (float*)take(nu * plan.shape.D * sizeof(float));
  w.edge_mask = (uint8_t*)take((size_t)plan.rows_in);
  w.slot = (int32_t*)take((size_t)plan.rows_in * sizeof(int32_t));
  // one-pass score kernel: statistics and partial o_bar of every work item, counters and flags
  if (plan.fused_items > 0) {
    w.fstats = (float*)take((size_t)plan.fused_items * plan.shape.R * sizeof(float));
    w.fo_part = (float*)take((size_t)plan.fused_items * plan.shape.D * sizeof(float));
    w.fsync = (unsigned int*)take(((size_t)kFusedSyncInts + plan.fused_items) * sizeof(unsigned int));
  }
  // exchange area of the selection by several workgroups per unit (one launch group at a time)
  w.sel_shared = (unsigned int*)take((size_t)std::min(plan.n_units, kInlineUnits) * kSelSharedInts * sizeof(unsigned int));
  w.unit_tab = (Unit*)take(plan.n_units > kInlineUnits ? (size_t)std::min(plan.n_units, kMaxGroupUnits) * sizeof(Unit) : 0);
  w.bytes = off;
  return w;
}

// Extra workspace of the per-query aggregation, laid out behind the ordinary one.
struct PerQueryWs {
  float* o_part;     // [a launch's chunks][R][D] partial outputs, then [a launch's chunks][R] sums of their weights
  uint16_t* o_hi;    // [n_units][R][D]  bf16 inputs: -2 o as a bf16 pair hi + lo
  uint16_t* o_lo;
  float* o_f32;      // [n_units][R][D]  fp32 inputs: o itself
  float* oo;         // [n_units][R]
  float* a_tok;      // [rows]  (kvs_step_per_query only)
  float* c_edge;     // [rows]
  size_t bytes;      // ordinary workspace included
};

PerQueryWs carve_per_query(const Plan& plan, void* base, Workspace* w) {
  *w = carve(plan, base);
  PerQueryWs q{};
  size_t off = w->bytes;
  auto take = [&](size_t bytes) {
    char* ptr = base ? (char*)base + off : nullptr;
    off += align_up(bytes);
    return (void*)ptr;
  };
  // (the chunks of the largest group; groups of a call that has to keep them smaller need less)
  long long max_chunks = 0;
  for (int first = 0, end; first < plan.n_units; first = end) {
    end = group_end(plan, first, plan.group_cap);
    long long c = 0;
    for (int u = first; u < end; ++u) c += plan.units[u].n_chunks;
    max_chunks = std::max(max_chunks, c);
  }
  const size_t rd = (size_t)plan.shape.R * plan.shape.D;
  q.o_part = (float*)take((size_t)max_chunks * (rd + plan.shape.R) * sizeof(float));
  if (plan.dtype == KVS_F32) {
    q.o_f32 = (float*)take((size_t)plan.n_units * rd * sizeof(float));
  } else {
    q.o_hi = (uint16_t*)take((size_t)plan.n_units * rd * sizeof(uint16_t));
    q.o_lo = (uint16_t*)take((size_t)plan.n_units * rd * sizeof(uint16_t));
  }
  q.oo = (float*)take((size_t)plan.n_units * plan.shape.R * sizeof(float));
  q.a_tok = (float*)take((size_t)plan.rows_in * sizeof(float));
  q.c_edge = (float*)take((size_t)plan.rows_in * sizeof(float));
  q.bytes = off;
  return q;
}

// The per-query kernels are bf16 MFMA kernels whose tiles hold 32 whole rows of a unit.
kvs_status check_per_query(const Plan& plan) {
  if (plan.dtype == KVS_F32) return KVS_OK;         // the fp32 kernels take any unit length
  for (const Unit& un : plan.units) {               // bf16: whole MFMA tiles of 32 rows
    if (un.len < 32) return KVS_ERR_INVALID_ARG;
  }
  return KVS_OK;
}

hipError_t per_query_norms(const Plan& plan, const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                           const void* V, const int32_t* counts_in, const Workspace& w, const PerQueryWs& q,
                           float* a_tok, float* c_edge, hipStream_t s) {
  if (plan.dtype == KVS_F32)
    return launch_per_query_norms_f32(tab, sh, Q, K, V, counts_in, w.c_row, q.o_part, q.o_f32, a_tok, c_edge, s);
  return launch_per_query_norms(tab, sh, Q, K, V, counts_in, w.c_row, q.o_part, q.o_hi, q.o_lo, q.oo, a_tok, c_edge, s);
}

struct Range {
  const void* p;
  size_t bytes;
  bool is_output;
};

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

kvs_status check_ranges(const std::vector<Range>& rs) {
  for (const Range& r : rs) {
    if (r.p == nullptr || !aligned16(r.p)) return KVS_ERR_INVALID_ARG;
  }
  for (size_t i = 0; i < rs.size(); ++i) {
    if (!rs[i].is_output) continue;
    for (size_t j = 0; j < rs.size(); ++j) {
      if (i == j) continue;
      const char* a0 = (const char*)rs[i].p;
      const char* b0 = (const char*)rs[j].p;
      if (a0 < b0 + rs[j].bytes && b0 < a0 + rs[i].bytes) return KVS_ERR_ALIAS;
    }
  }
  return KVS_OK;
}

kvs_status check_ws(const Plan& plan, const void* ws, size_t ws_bytes, Workspace* out, void* ws_mut) {
  if (ws == nullptr || ((uintptr_t)ws % kAlign) != 0) return KVS_ERR_WORKSPACE;
  *out = carve(plan, ws_mut);
  if (ws_bytes < out->bytes) return KVS_ERR_WORKSPACE;
  return KVS_OK;
}

// The decode workspace: the chunks' partial results, then (calls of more than kInlineUnits units) the descriptors of
// a launch group.
size_t decode_partial_bytes(const Plan& plan) {
  return align_up((size_t)plan.n_units * kMaxChunks * plan.shape.R * (plan.shape.D + 2) * sizeof(float));
}
size_t decode_table_bytes(const Plan& plan) {
  return plan.n_units > kInlineUnits ? align_up((size_t)std::min(plan.n_units, kMaxGroupUnits) * sizeof(Unit)) : 0;
}

// An entry point whose workspace is optional: with one that is usable, its groups may keep their descriptors there.
// Returns the bytes of it that the call may write (0: none).
size_t adopt_optional_ws(Plan& plan, void* ws, size_t ws_bytes) {
  if (ws == nullptr || ((uintptr_t)ws % kAlign) != 0) return 0;
  const Workspace w = carve(plan, ws);
  if (ws_bytes < w.bytes) return 0;
  plan.dev_table = w.unit_tab;
  return w.bytes;
}

// Compute units of the current device (asked once per device).
int compute_units() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Calls f(table, shape) for every launch group (see group_end).
// split_select: the caller hands the launchers an exchange area, so a unit's selection may take several workgroups.
template <typename F>
kvs_status for_each_group(const Plan& plan, F&& f, bool split_select = false) {
  // An error that the calling thread's earlier HIP calls left pending is not this call's: it is dropped here,
  // so that what the launchers read after their launches is theirs.
  (void)hipGetLastError();
  const int split_mode = split_select ? debug_switch(KVS_DEBUG_SELECT_SPLIT) : 1;
  const int n_cus = split_mode == 1 ? 0 : compute_units();
  // A group of more than kInlineUnits units needs memory for its descriptors.  Where a test asks for every unit's
  // selection to be spread over workgroups, the exchange area's kInlineUnits entries bound the group as well (left
  // to itself the library spreads a selection only in launches of a few units).
  int cap = plan.dev_table != nullptr ? plan.group_cap : std::min(plan.group_cap, kInlineUnits);
  if (split_mode >= 2) cap = std::min(cap, kInlineUnits);
  std::vector<Unit> units;
  for (int first = 0, end; first < plan.n_units; first = end) {
    end = group_end(plan, first, cap);
    UnitTable tab;
    std::memset(&tab, 0, sizeof(tab));
    tab.n_units = end - first;
    units.assign(plan.units.begin() + first, plan.units.begin() + end);
    int chunks = 0, mblocks = 0, ochunks = 0, fitems = 0, sparts = 0;
    long long rows = 0;
    for (Unit& un : units) {
      un.s_base = sparts;
      sparts += select_parts(un, plan.shape, tab.n_units, n_cus, split_mode);
      un.chunk_base = chunks;
      un.m_base = mblocks;
      un.o_base = ochunks;
      un.f_base = fitems;
      fitems += fused_chunks(un.len, plan.shape.D);
      ochunks += obar_chunks(un.len);
      chunks += un.n_chunks;
      mblocks += (un.len + kMergeTokens - 1) / kMergeTokens;
      rows += un.len;
    }
    tab.total_chunks = chunks;
    tab.total_mblocks = mblocks;
    tab.total_ochunks = ochunks;
    tab.total_fitems = fitems;
    tab.total_sparts = sparts;
    Shape sh = plan.shape;
    sh.stream = 2 * rows * sh.D * (long long)plan.elt > kStreamBytes;
    hipError_t e = hipSuccess;
    if (tab.n_units <= kInlineUnits) {
      std::copy(units.begin(), units.end(), tab.u);
    } else {
      tab.host = units.data();
      tab.ext = plan.dev_table;
      e = launch_unit_table(units.data(), tab.n_units, plan.dev_table, plan.stream);
    }
    if (e == hipSuccess) e = f(tab, sh);
    if (e != hipSuccess) {
      if (debug_switch(KVS_DEBUG_VERBOSE)) {
        std::fprintf(stderr, "libkvs: launch failed in the group of units %d..%d: %s\n", first, first + tab.n_units - 1,
                     hipGetErrorString(e));
      }
      return KVS_ERR_DEVICE;
    }
  }
  return KVS_OK;
}

}  // namespace

int select_parts(const Unit& un, const Shape& sh, int n_units, int n_cus, int mode) {
  const int r = un.len - un.n_out;
  const int E = (un.len - 2 - sh.n_recent) - sh.n_sink + 1;      // eligible edges
  if (mode == 1 || r <= 0 || E < 64) return 1;
  const int groups = (E + 6) / 4 + 1;                            // upper bound of the kernel's group count
  const int fit = (groups + kSelPartKeys / 4 - 1) / (kSelPartKeys / 4);   // fewest parts whose keys fit their LDS
  // one select workgroup per CU, so that the parts of a launch run together (a test may ask for more)
  // A launch of many units keeps the chip busy with one workgroup per unit, and on a chip shared with another
  // stream's kernels its parts would wait for each other's turn (64 units at 4 parts each: 67.0 us per layer of the
  // two-stream headline run against 65.6): the parts are for launches that leave most compute units idle.
  // (Splitting only the units that are too long for one workgroup's key cache was measured on the ragged batch,
  // 64 units of 4 K to 64 K tokens per launch: the launch of selection and pass over V took 117 us against 108,
  // because the selection is hidden beside that pass anyway and the parts take compute units from it.)
  if (mode == 0 && n_cus / n_units < 8) return 1;
  const int most = mode >= 2 ? kSelMaxParts : (n_cus / n_units < kSelMaxParts ? n_cus / n_units : kSelMaxParts);
  const int min_keys = mode >= 2 ? 64 : kSelMinPartKeys;
  int P = (E + min_keys - 1) / min_keys;
  if (P > most) P = most;
  if (P < 2 || P < fit) return 1;                                // not worth it, or too long for the parts it may have
  return P;
}

hipError_t launch_score(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* Q, const void* K,
                        const int32_t* counts_in, float* alpha_bar, const Workspace& ws, hipStream_t stream,
                        const void* V, int* o_layout) {
  // KVS_DEBUG_SCORE_PATH forces the vector-ALU kernels (used by the tests to cover both paths).
  const bool force_valu = debug_switch(KVS_DEBUG_SCORE_PATH) == 1;
  if (o_layout) *o_layout = 0;
  const bool wants_o = V != nullptr && o_layout != nullptr;
  // Windows of 65..128 bf16 rows can take the one-pass kernel, which reads K once, keeps it in LDS between the
  // statistics and the alpha_bar phase and carries the pass over V along (it needs V: callers that only want
  // alpha_bar take the two sweeps).  It is correct and saves a third of the score phase's traffic, but on this
  // chip it is slower than the two sweeps (see the measurements at the kernel), so it runs on request only:
  // KVS_DEBUG_SCORE_FUSED = 2.
  if (!force_valu && wants_o && ws.fsync != nullptr && debug_switch(KVS_DEBUG_SCORE_FUSED) == 2 &&
      score_fused_supported(tab, sh, dt)) {
    *o_layout = 2;
    return launch_score_fused(tab, sh, Q, K, V, counts_in, alpha_bar, ws, stream);
  }
  // The pass over V rides along in sweep 1 when the launch is a large one (the streaming policy's threshold):
  // the edge selection then runs as a short launch of its own, one CU per unit, which costs less than the
  // separate pass over V saves (measured at 64 units of the headline shape: 199 against 226 us for sweep 1,
  // the pass over V and the selection).  A small launch keeps the selection hidden beside the pass over V
  // (8 units: 38 against 45 us).  KVS_DEBUG_FUSE_OBAR forces one or the other.
  if (!force_valu && score_mfma_supported(tab, sh, dt)) {
    const int fuse = debug_switch(KVS_DEBUG_FUSE_OBAR);
    // (The selection of a unit too long for the select kernel's LDS cache of keys takes several times longer when one
    // workgroup does it, 51 us at 65536 tokens: such launches keep it hidden beside the pass over V, unless the
    // unit's selection is spread over several workgroups.)
    int longest = 0;
    for (int i = 0; i < tab.n_units; ++i) {
      const int parts = (i + 1 < tab.n_units ? tab.unit(i + 1).s_base : tab.total_sparts) - tab.unit(i).s_base;
      if (parts <= 1) longest = std::max(longest, tab.unit(i).len);
    }
    bool want = sh.stream != 0 && longest <= kSelUnitKeys;
    if (fuse == 1) want = false;
    if (fuse == 2) want = true;
    const bool with_v = wants_o && score_mfma_takes_values(sh, dt) && want;
    if (with_v) *o_layout = 1;
    return launch_score_mfma(tab, sh, dt, Q, K, counts_in, alpha_bar, ws, with_v ? V : nullptr, stream);
  }
  return launch_score_valu(tab, sh, dt, Q, K, counts_in, alpha_bar, ws, stream);
}

}  // namespace kvs

using namespace kvs;

extern "C" {

kvs_status kvs_workspace_size(const kvs_problem* p, size_t* bytes) {
  if (bytes == nullptr) return KVS_ERR_INVALID_ARG;
  Plan plan;
  const kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  *bytes = carve(plan, nullptr).bytes;
  return KVS_OK;
}

kvs_status kvs_score(const kvs_problem* p, const void* Q, const void* K, const void* V, float* alpha_bar,
                     float* o_bar, void* ws, size_t ws_bytes, void* hip_stream) {
  return kvs_score_counts(p, Q, K, V, nullptr, alpha_bar, o_bar, ws, ws_bytes, hip_stream);
}

kvs_status kvs_score_counts(const kvs_problem* p, const void* Q, const void* K, const void* V,
                            const int32_t* counts_in, float* alpha_bar, float* o_bar, void* ws, size_t ws_bytes,
                            void* hip_stream) {
  Plan plan;
  kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  Workspace w;
  if ((st = check_ws(plan, ws, ws_bytes, &w, ws)) != KVS_OK) return st;
  const size_t kv = (size_t)plan.rows_in * plan.shape.D * plan.elt;
  const size_t nu = (size_t)plan.n_units;
  std::vector<Range> rs = {{Q, nu * plan.shape.R * plan.shape.D * plan.elt, false},
                           {K, kv, false},
                           {V, kv, false},
                           {alpha_bar, (size_t)plan.rows_in * 4, true},
                           {o_bar, nu * plan.shape.D * 4, true},
                           {ws, w.bytes, true}};
  if (counts_in) rs.push_back({counts_in, (size_t)plan.rows_in * 4, false});
  if ((st = check_ranges(rs)) != KVS_OK) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  plan.dev_table = w.unit_tab;
  plan.stream = s;
  return for_each_group(plan, [&](const UnitTable& tab, const Shape& sh) {
    int o_layout = 0;
    hipError_t e = launch_score(tab, sh, plan.dtype, Q, K, counts_in, alpha_bar, w, s, V, &o_layout);
    if (e != hipSuccess) return e;
    Shape sh2 = sh;
    sh2.o_from_score = o_layout;
    if (o_layout == 0) {
      e = launch_select_obar(tab, sh, plan.dtype, false, alpha_bar, nullptr, nullptr, V, counts_in, w.o_part, s);
      if (e != hipSuccess) return e;
    }
    return launch_obar_reduce(tab, sh2, o_layout == 2 ? w.fo_part : w.o_part, o_bar, s);
  });
}

kvs_status kvs_select(const kvs_problem* p, const float* alpha_bar, uint8_t* edge_mask, int32_t* slot_of_token,
                      void* ws, size_t ws_bytes, void* hip_stream) {
  Plan plan;
  kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  std::vector<Range> rs = {{alpha_bar, (size_t)plan.rows_in * 4, false},
                           {edge_mask, (size_t)plan.rows_in, true},
                           {slot_of_token, (size_t)plan.rows_in * 4, true}};
  // The workspace is optional here: with one (of kvs_workspace_size bytes) a long unit's selection may be spread
  // over several workgroups, which meet through it; without one every unit takes a single workgroup.
  Workspace w{};
  const bool with_ws = ws != nullptr && ((uintptr_t)ws % kAlign) == 0 && ws_bytes >= carve(plan, nullptr).bytes;
  if (with_ws) {
    w = carve(plan, ws);
    rs.push_back({ws, w.bytes, true});
  }
  if ((st = check_ranges(rs)) != KVS_OK) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  if (with_ws) plan.dev_table = w.unit_tab;
  plan.stream = s;
  return for_each_group(plan, [&](const UnitTable& tab, const Shape& sh) {
    if (tab.total_sparts != tab.n_units) {      // (the score kernels clear the area when they run before the selection)
      const hipError_t e = launch_select_clear(tab, w.sel_shared, s);
      if (e != hipSuccess) return e;
    }
    return launch_select_obar(tab, sh, plan.dtype, true, alpha_bar, edge_mask, slot_of_token, nullptr,
                              nullptr, nullptr, s, nullptr, nullptr, w.sel_shared);
  }, /*split_select=*/with_ws);
}

kvs_status kvs_merge_compact(const kvs_problem* p, const void* K, const void* V, const float* alpha_bar,
                             const float* o_bar, const uint8_t* edge_mask, const int32_t* slot_of_token,
                             void* K_out, void* V_out, int32_t* counts_out, void* ws, size_t ws_bytes,
                             void* hip_stream) {
  return kvs_merge_compact_counts(p, K, V, nullptr, alpha_bar, o_bar, edge_mask, slot_of_token, K_out, V_out,
                                  counts_out, ws, ws_bytes, hip_stream);
}

kvs_status kvs_merge_compact_counts(const kvs_problem* p, const void* K, const void* V, const int32_t* counts_in,
                                    const float* alpha_bar, const float* o_bar, const uint8_t* edge_mask,
                                    const int32_t* slot_of_token, void* K_out, void* V_out, int32_t* counts_out,
                                    void* ws, size_t ws_bytes, void* hip_stream) {
  Plan plan;
  kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  const size_t ws_used = adopt_optional_ws(plan, ws, ws_bytes);
  const size_t kv = (size_t)plan.rows_in * plan.shape.D * plan.elt;
  const size_t kvo = (size_t)plan.rows_out * plan.shape.D * plan.elt;
  std::vector<Range> rs = {{K, kv, false},
                           {V, kv, false},
                           {alpha_bar, (size_t)plan.rows_in * 4, false},
                           {o_bar, (size_t)plan.n_units * plan.shape.D * 4, false},
                           {edge_mask, (size_t)plan.rows_in, false},
                           {slot_of_token, (size_t)plan.rows_in * 4, false},
                           {K_out, kvo, true},
                           {V_out, kvo, true},
                           {counts_out, (size_t)plan.rows_out * 4, true}};
  if (counts_in) rs.push_back({counts_in, (size_t)plan.rows_in * 4, false});
  if (ws_used) rs.push_back({ws, ws_used, true});
  if ((st = check_ranges(rs)) != KVS_OK) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  plan.stream = s;
  return for_each_group(plan, [&](const UnitTable& tab, const Shape& sh) {
    return launch_merge(tab, sh, plan.dtype, K, V, counts_in, alpha_bar, o_bar, nullptr, edge_mask, slot_of_token,
                        K_out, V_out, counts_out, s);
  });
}

kvs_status kvs_step(const kvs_problem* p, const void* Q, const void* K, const void* V, void* K_out, void* V_out,
                    int32_t* counts_out, int32_t* slot_of_token_out, uint8_t* edge_mask_out, void* ws,
                    size_t ws_bytes, void* hip_stream) {
  return kvs_step_counts(p, Q, K, V, nullptr, K_out, V_out, counts_out, slot_of_token_out, edge_mask_out, ws,
                         ws_bytes, hip_stream);
}

// Pointer, alignment and overlap checks of a step's arguments; ws may be null (then it is left out).
static kvs_status check_step_ranges(const Plan& plan, const void* Q, const void* K, const void* V,
                                    const int32_t* counts_in, void* K_out, void* V_out, int32_t* counts_out,
                                    int32_t* slot_of_token_out, uint8_t* edge_mask_out, void* ws, size_t ws_used) {
  const size_t kv = (size_t)plan.rows_in * plan.shape.D * plan.elt;
  const size_t kvo = (size_t)plan.rows_out * plan.shape.D * plan.elt;
  std::vector<Range> rs = {{Q, (size_t)plan.n_units * plan.shape.R * plan.shape.D * plan.elt, false},
                           {K, kv, false},
                           {V, kv, false},
                           {K_out, kvo, true},
                           {V_out, kvo, true},
                           {counts_out, (size_t)plan.rows_out * 4, true}};
  if (ws) rs.push_back({ws, ws_used, true});
  if (slot_of_token_out) rs.push_back({slot_of_token_out, (size_t)plan.rows_in * 4, true});
  if (edge_mask_out) rs.push_back({edge_mask_out, (size_t)plan.rows_in, true});
  if (counts_in) rs.push_back({counts_in, (size_t)plan.rows_in * 4, false});
  return check_ranges(rs);
}

// kvs_step_counts with the workspace given either by the caller (ws, ws_bytes) or, for kvs_step_static, by
// `fixed_ws` (then ws_bytes is its capacity and the caller's argument checks have run before any device call).
static kvs_status step_with_workspace(Plan& plan, const void* Q, const void* K, const void* V,
                                      const int32_t* counts_in, void* K_out, void* V_out, int32_t* counts_out,
                                      int32_t* slot_of_token_out, uint8_t* edge_mask_out, void* ws, size_t ws_bytes,
                                      void* hip_stream) {
  kvs_status st;
  Workspace w;
  if ((st = check_ws(plan, ws, ws_bytes, &w, ws)) != KVS_OK) return st;
  if ((st = check_step_ranges(plan, Q, K, V, counts_in, K_out, V_out, counts_out, slot_of_token_out, edge_mask_out, ws,
                              w.bytes)) != KVS_OK) {
    return st;
  }

  uint8_t* mask = edge_mask_out ? edge_mask_out : w.edge_mask;
  int32_t* slot = slot_of_token_out ? slot_of_token_out : w.slot;
  hipStream_t s = (hipStream_t)hip_stream;
  plan.dev_table = w.unit_tab;
  plan.stream = s;
  return for_each_group(plan, [&](const UnitTable& tab, const Shape& sh) {
    int o_layout = 0;
    hipError_t e = launch_score(tab, sh, plan.dtype, Q, K, counts_in, w.alpha_bar, w, s, V, &o_layout);
    if (e != hipSuccess) return e;
    Shape sh2 = sh;
    sh2.o_from_score = o_layout;
    if (o_layout == 2) {
      // the one-pass kernel leaves one partial o_bar per work item (a few hundred per unit): they are added up by
      // one more workgroup per unit beside the selection, and the merge pass takes the finished o_bar
      e = launch_select_obar(tab, sh2, plan.dtype, true, w.alpha_bar, mask, slot, nullptr, counts_in, nullptr, s,
                             w.fo_part, w.o_bar, w.sel_shared);
      if (e != hipSuccess) return e;
      return launch_merge(tab, sh2, plan.dtype, K, V, counts_in, w.alpha_bar, w.o_bar, nullptr, mask, slot, K_out,
                          V_out, counts_out, s);
    }
    e = launch_select_obar(tab, sh, plan.dtype, true, w.alpha_bar, mask, slot, o_layout ? nullptr : V, counts_in,
                           w.o_part, s, nullptr, nullptr, w.sel_shared);
    if (e != hipSuccess) return e;
    return launch_merge(tab, sh2, plan.dtype, K, V, counts_in, w.alpha_bar, nullptr, w.o_part, mask, slot, K_out,
                        V_out, counts_out, s);
  }, /*split_select=*/true);
}

kvs_status kvs_step_counts(const kvs_problem* p, const void* Q, const void* K, const void* V, const int32_t* counts_in,
                           void* K_out, void* V_out, int32_t* counts_out, int32_t* slot_of_token_out,
                           uint8_t* edge_mask_out, void* ws, size_t ws_bytes, void* hip_stream) {
  Plan plan;
  const kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  return step_with_workspace(plan, Q, K, V, counts_in, K_out, V_out, counts_out, slot_of_token_out, edge_mask_out, ws,
                             ws_bytes, hip_stream);
}

// ---- kvs_step_static: the step for callers that cannot allocate.  Its workspace is this array: one copy per GPU
// that runs the library, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address it yields (per device) is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[KVS_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];      // device address of `scratch` on every device that has asked for it

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
kvs_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KVS_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr) {
      if (debug_switch(KVS_DEBUG_VERBOSE)) {
        std::fprintf(stderr, "libkvs: hipGetSymbolAddress(scratch) failed on device %d: %s\n", dev, hipGetErrorString(e));
      }
      return KVS_ERR_DEVICE;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return KVS_OK;
}
}  // namespace

kvs_status kvs_step_static(const kvs_problem* p, const void* Q, const void* K, const void* V, const int32_t* counts_in,
                           void* K_out, void* V_out, int32_t* counts_out, int32_t* slot_of_token_out,
                           uint8_t* edge_mask_out, void* hip_stream) {
  Plan plan;
  kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  // the size check needs no device: a problem beyond the array is refused before anything touches the GPU
  if (carve(plan, nullptr).bytes > (size_t)KVS_STATIC_SCRATCH_BYTES) return KVS_ERR_WORKSPACE;
  if ((st = check_step_ranges(plan, Q, K, V, counts_in, K_out, V_out, counts_out, slot_of_token_out, edge_mask_out,
                              nullptr, 0)) != KVS_OK) {
    return st;
  }
  void* ws = nullptr;
  if ((st = static_scratch(&ws)) != KVS_OK) return st;
  return step_with_workspace(plan, Q, K, V, counts_in, K_out, V_out, counts_out, slot_of_token_out, edge_mask_out, ws,
                             (size_t)KVS_STATIC_SCRATCH_BYTES, hip_stream);
}

kvs_status kvs_per_query_workspace_size(const kvs_problem* p, size_t* bytes) {
  if (bytes == nullptr) return KVS_ERR_INVALID_ARG;
  Plan plan;
  kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  if ((st = check_per_query(plan)) != KVS_OK) return st;
  Workspace w;
  *bytes = carve_per_query(plan, nullptr, &w).bytes;
  return KVS_OK;
}

kvs_status kvs_sensitivity(const kvs_problem* p, const void* Q, const void* K, const void* V, float* alpha_bar,
                           float* a_tok, float* c_edge, void* ws, size_t ws_bytes, void* hip_stream) {
  return kvs_sensitivity_counts(p, Q, K, V, nullptr, alpha_bar, a_tok, c_edge, ws, ws_bytes, hip_stream);
}

kvs_status kvs_sensitivity_counts(const kvs_problem* p, const void* Q, const void* K, const void* V,
                                  const int32_t* counts_in, float* alpha_bar, float* a_tok, float* c_edge, void* ws,
                                  size_t ws_bytes, void* hip_stream) {
  Plan plan;
  kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  if ((st = check_per_query(plan)) != KVS_OK) return st;
  if (ws == nullptr || ((uintptr_t)ws % kAlign) != 0) return KVS_ERR_WORKSPACE;
  Workspace w;
  const PerQueryWs q = carve_per_query(plan, ws, &w);
  if (ws_bytes < q.bytes) return KVS_ERR_WORKSPACE;
  const size_t kv = (size_t)plan.rows_in * plan.shape.D * plan.elt;
  const size_t rows4 = (size_t)plan.rows_in * 4;
  std::vector<Range> rs = {{Q, (size_t)plan.n_units * plan.shape.R * plan.shape.D * plan.elt, false},
                           {K, kv, false},
                           {V, kv, false},
                           {alpha_bar, rows4, true},
                           {a_tok, rows4, true},
                           {c_edge, rows4, true},
                           {ws, q.bytes, true}};
  if (counts_in) rs.push_back({counts_in, rows4, false});
  if ((st = check_ranges(rs)) != KVS_OK) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  plan.dev_table = w.unit_tab;
  plan.stream = s;
  return for_each_group(plan, [&](const UnitTable& tab, const Shape& sh) {
    hipError_t e = launch_score(tab, sh, plan.dtype, Q, K, counts_in, alpha_bar, w, s);
    if (e != hipSuccess) return e;
    return per_query_norms(plan, tab, sh, Q, K, V, counts_in, w, q, a_tok, c_edge, s);
  });
}

kvs_status kvs_merge_compact_norms(const kvs_problem* p, const void* K, const void* V, const float* a_tok,
                                   const float* c_edge, const uint8_t* edge_mask, const int32_t* slot_of_token,
                                   void* K_out, void* V_out, int32_t* counts_out, void* ws, size_t ws_bytes,
                                   void* hip_stream) {
  return kvs_merge_compact_norms_counts(p, K, V, nullptr, a_tok, c_edge, edge_mask, slot_of_token, K_out, V_out,
                                        counts_out, ws, ws_bytes, hip_stream);
}

kvs_status kvs_merge_compact_norms_counts(const kvs_problem* p, const void* K, const void* V, const int32_t* counts_in,
                                          const float* a_tok, const float* c_edge, const uint8_t* edge_mask,
                                          const int32_t* slot_of_token, void* K_out, void* V_out, int32_t* counts_out,
                                          void* ws, size_t ws_bytes, void* hip_stream) {
  Plan plan;
  kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  const size_t ws_used = adopt_optional_ws(plan, ws, ws_bytes);
  const size_t kv = (size_t)plan.rows_in * plan.shape.D * plan.elt;
  const size_t kvo = (size_t)plan.rows_out * plan.shape.D * plan.elt;
  std::vector<Range> rs = {{K, kv, false},
                           {V, kv, false},
                           {a_tok, (size_t)plan.rows_in * 4, false},
                           {c_edge, (size_t)plan.rows_in * 4, false},
                           {edge_mask, (size_t)plan.rows_in, false},
                           {slot_of_token, (size_t)plan.rows_in * 4, false},
                           {K_out, kvo, true},
                           {V_out, kvo, true},
                           {counts_out, (size_t)plan.rows_out * 4, true}};
  if (counts_in) rs.push_back({counts_in, (size_t)plan.rows_in * 4, false});
  if (ws_used) rs.push_back({ws, ws_used, true});
  if ((st = check_ranges(rs)) != KVS_OK) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  plan.stream = s;
  return for_each_group(plan, [&](const UnitTable& tab, const Shape& sh) {
    return launch_merge_norms(tab, sh, plan.dtype, K, V, counts_in, a_tok, c_edge, edge_mask, slot_of_token, K_out,
                              V_out, counts_out, s);
  });
}

kvs_status kvs_step_per_query(const kvs_problem* p, const void* Q, const void* K, const void* V, void* K_out,
                              void* V_out, int32_t* counts_out, int32_t* slot_of_token_out, uint8_t* edge_mask_out,
                              void* ws, size_t ws_bytes, void* hip_stream) {
  return kvs_step_per_query_counts(p, Q, K, V, nullptr, K_out, V_out, counts_out, slot_of_token_out, edge_mask_out, ws,
                                   ws_bytes, hip_stream);
}

kvs_status kvs_step_per_query_counts(const kvs_problem* p, const void* Q, const void* K, const void* V,
                                     const int32_t* counts_in, void* K_out, void* V_out, int32_t* counts_out,
                                     int32_t* slot_of_token_out, uint8_t* edge_mask_out, void* ws, size_t ws_bytes,
                                     void* hip_stream) {
  Plan plan;
  kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  if ((st = check_per_query(plan)) != KVS_OK) return st;
  if (ws == nullptr || ((uintptr_t)ws % kAlign) != 0) return KVS_ERR_WORKSPACE;
  Workspace w;
  const PerQueryWs q = carve_per_query(plan, ws, &w);
  if (ws_bytes < q.bytes) return KVS_ERR_WORKSPACE;
  const size_t kv = (size_t)plan.rows_in * plan.shape.D * plan.elt;
  const size_t kvo = (size_t)plan.rows_out * plan.shape.D * plan.elt;
  std::vector<Range> rs = {{Q, (size_t)plan.n_units * plan.shape.R * plan.shape.D * plan.elt, false},
                           {K, kv, false},
                           {V, kv, false},
                           {K_out, kvo, true},
                           {V_out, kvo, true},
                           {counts_out, (size_t)plan.rows_out * 4, true},
                           {ws, q.bytes, true}};
  if (slot_of_token_out) rs.push_back({slot_of_token_out, (size_t)plan.rows_in * 4, true});
  if (edge_mask_out) rs.push_back({edge_mask_out, (size_t)plan.rows_in, true});
  if (counts_in) rs.push_back({counts_in, (size_t)plan.rows_in * 4, false});
  if ((st = check_ranges(rs)) != KVS_OK) return st;
  uint8_t* mask = edge_mask_out ? edge_mask_out : w.edge_mask;
  int32_t* slot = slot_of_token_out ? slot_of_token_out : w.slot;
  hipStream_t s = (hipStream_t)hip_stream;
  plan.dev_table = w.unit_tab;
  plan.stream = s;
  return for_each_group(plan, [&](const UnitTable& tab, const Shape& sh) {
    hipError_t e = launch_score(tab, sh, plan.dtype, Q, K, counts_in, w.alpha_bar, w, s);
    if (e != hipSuccess) return e;
    e = launch_select_obar(tab, sh, plan.dtype, true, w.alpha_bar, mask, slot, nullptr, nullptr, nullptr, s, nullptr,
                           nullptr, w.sel_shared);
    if (e != hipSuccess) return e;
    e = per_query_norms(plan, tab, sh, Q, K, V, counts_in, w, q, q.a_tok, q.c_edge, s);
    if (e != hipSuccess) return e;
    return launch_merge_norms(tab, sh, plan.dtype, K, V, counts_in, q.a_tok, q.c_edge, mask, slot, K_out, V_out,
                              counts_out, s);
  }, /*split_select=*/true);
}

kvs_status kvs_decode_workspace_size(const kvs_problem* p, size_t* bytes) {
  if (bytes == nullptr) return KVS_ERR_INVALID_ARG;
  Plan plan;
  const kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  if (plan.shape.R > KVS_MAX_DECODE_ROWS) return KVS_ERR_INVALID_ARG;
  *bytes = decode_partial_bytes(plan) + decode_table_bytes(plan);
  return KVS_OK;
}

kvs_status kvs_decode_attention(const kvs_problem* p, const void* Q, const void* K, const void* V,
                                const int32_t* counts, float* out, void* ws, size_t ws_bytes, void* hip_stream) {
  Plan plan;
  kvs_status st = make_plan(p, &plan);
  if (st != KVS_OK) return st;
  if (plan.shape.R > KVS_MAX_DECODE_ROWS) return KVS_ERR_INVALID_ARG;
  const size_t need = decode_partial_bytes(plan) + decode_table_bytes(plan);
  if (ws == nullptr || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < need) return KVS_ERR_WORKSPACE;
  const size_t kv = (size_t)plan.rows_in * plan.shape.D * plan.elt;
  const size_t qo = (size_t)plan.n_units * plan.shape.R * plan.shape.D;
  std::vector<Range> rs = {{Q, qo * plan.elt, false}, {K, kv, false}, {V, kv, false},
                           {out, qo * sizeof(float), true}, {ws, need, true}};
  if (counts) rs.push_back({counts, (size_t)plan.rows_in * 4, false});
  if ((st = check_ranges(rs)) != KVS_OK) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  if (decode_table_bytes(plan)) plan.dev_table = (Unit*)((char*)ws + decode_partial_bytes(plan));
  plan.stream = s;
  return for_each_group(plan, [&](const UnitTable& tab, const Shape& sh) {
    return launch_decode(tab, sh, plan.dtype, Q, K, V, counts, (float*)ws, out, s);
  });
}

int kvs_debug_set(int which, int value) {
  if (which < 0 || which >= KVS_DEBUG_N_SWITCHES || value < 0) return -1;
  return g_switch[which].exchange(value, std::memory_order_relaxed);
}

int kvs_debug_get(int which) {
  if (which < 0 || which >= KVS_DEBUG_N_SWITCHES) return -1;
  return debug_switch((kvs_debug_switch)which);
}

const char* kvs_status_str(kvs_status s) {
  switch (s) {
    case KVS_OK: return "ok";
    case KVS_ERR_INVALID_ARG: return "invalid argument";
    case KVS_ERR_DTYPE: return "unsupported dtype";
    case KVS_ERR_BUDGET: return "budget too small for n_sink + n_recent";
    case KVS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case KVS_ERR_ALIAS: return "an output overlaps another buffer";
    case KVS_ERR_DEVICE: return "HIP launch failed";
  }
  return "unknown status";
}

int kvs_version(void) { return KVS_VERSION; }

}  // extern "C"
