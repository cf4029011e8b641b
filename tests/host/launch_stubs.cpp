// Host-only stand-ins for the kernel launchers of libkvs: every launch "succeeds" without touching a GPU, so that
// the host layer (argument validation, workspace carve-up, unit tables, launch sequencing in kvs_api.hip) can run
// to the end of a call on the CPU, under AddressSanitizer and UndefinedBehaviorSanitizer.  Test infrastructure.
#include "kvs_device.h"

namespace kvs {

static int g_launches = 0;
int stub_launches() { return g_launches; }

static hipError_t ok() { ++g_launches; return hipSuccess; }

// what a launcher may assume about its table: checked here so that a wrong table fails the sanitizer run
static const Unit* g_written = nullptr;   // where the last launch_unit_table put its descriptors, and how many
static int g_written_n = 0;

static void check_table(const UnitTable& tab) {
  if (tab.n_units < 1 || tab.n_units > kMaxGroupUnits) __builtin_trap();
  // a group beyond the inline descriptors must have had its descriptors written, to where the kernels will look
  if (tab.n_units > kInlineUnits) {
    if (tab.ext == nullptr || tab.host == nullptr || tab.ext != g_written || tab.n_units != g_written_n) __builtin_trap();
  } else if (tab.ext != nullptr || tab.host != nullptr) {
    __builtin_trap();
  }
  long long tokens = 0;
  for (int i = 0; i + 1 < tab.n_units; ++i) tokens += tab.unit(i).len;
  if (tab.n_units > kInlineUnits && tokens >= kGroupTokens) __builtin_trap();   // the group was full before its last unit
  int chunks = 0, mblocks = 0, ochunks = 0;
  for (int i = 0; i < tab.n_units; ++i) {
    const Unit u = tab.unit(i);
    if (u.len < 1 || u.n_out < 1 || u.n_out > u.len) __builtin_trap();
    if (u.chunk_len % kWave != 0 || u.n_chunks < 1 || u.n_chunks > kMaxChunks) __builtin_trap();
    if ((long long)u.chunk_len * u.n_chunks < u.len) __builtin_trap();
    if (u.chunk_base != chunks || u.m_base != mblocks || u.o_base != ochunks) __builtin_trap();
    chunks += u.n_chunks;
    mblocks += (u.len + kMergeTokens - 1) / kMergeTokens;
    ochunks += obar_chunks(u.len);
  }
  if (tab.total_chunks != chunks || tab.total_mblocks != mblocks || tab.total_ochunks != ochunks) __builtin_trap();
  for (int i = 0; i < tab.n_units; ++i) {          // select workgroups: one or several per unit, in unit order
    const int next = i + 1 < tab.n_units ? tab.unit(i + 1).s_base : tab.total_sparts;
    const int parts = next - tab.unit(i).s_base;
    if (tab.unit(i).s_base < i || parts < 1 || parts > kSelMaxParts) __builtin_trap();
    if (parts > 1 && tab.n_units > kInlineUnits) __builtin_trap();   // the exchange area has kInlineUnits entries
  }
}

hipError_t launch_unit_table(const Unit* units, int n_units, Unit* dst, hipStream_t) {
  if (units == nullptr || dst == nullptr || n_units <= kInlineUnits || n_units > kMaxGroupUnits) __builtin_trap();
  volatile long long touch = 0;
  for (int i = 0; i < n_units; ++i) touch = touch + units[i].len;   // (readable to its end, for the sanitizer)
  g_written = dst;
  g_written_n = n_units;
  return ok();
}
hipError_t launch_score_finalize(const UnitTable& tab, const Shape&, const Workspace&, hipStream_t) { check_table(tab); return ok(); }
hipError_t launch_score_valu(const UnitTable& tab, const Shape&, kvs_dtype, const void*, const void*, const int32_t*,
                             float*, const Workspace&, hipStream_t) { check_table(tab); return ok(); }
hipError_t launch_score_mfma(const UnitTable& tab, const Shape&, kvs_dtype, const void*, const void*, const int32_t*,
                             float*, const Workspace&, const void*, hipStream_t) { check_table(tab); return ok(); }
bool score_mfma_supported(const UnitTable& tab, const Shape& sh, kvs_dtype) {
  if (sh.R < 4) return false;
  for (int i = 0; i < tab.n_units; ++i) if (tab.unit(i).len < 32) return false;
  return true;
}
bool score_mfma_takes_values(const Shape& sh, kvs_dtype dt) { return dt == KVS_BF16 && sh.R > 64; }
bool score_fused_supported(const UnitTable&, const Shape& sh, kvs_dtype dt) { return dt == KVS_BF16 && sh.R > 64 && sh.R <= 128; }
hipError_t launch_score_fused(const UnitTable& tab, const Shape&, const void*, const void*, const void*, const int32_t*,
                              float*, const Workspace& ws, hipStream_t) {
  check_table(tab);
  if (ws.fstats == nullptr || ws.fo_part == nullptr || ws.fsync == nullptr) __builtin_trap();
  return ok();
}
hipError_t launch_select_obar(const UnitTable& tab, const Shape&, kvs_dtype, bool, const float*, uint8_t*, int32_t*,
                              const void*, const int32_t*, float*, hipStream_t, const float*, float*, unsigned int* sel_shared) {
  check_table(tab);
  if (tab.total_sparts != tab.n_units && sel_shared == nullptr) __builtin_trap();
  return ok();
}
hipError_t launch_select_clear(const UnitTable& tab, unsigned int* sel_shared, hipStream_t) {
  check_table(tab);
  if (sel_shared == nullptr) __builtin_trap();
  return ok();
}
hipError_t launch_obar_reduce(const UnitTable& tab, const Shape&, const float*, float*, hipStream_t) { check_table(tab); return ok(); }
hipError_t launch_merge(const UnitTable& tab, const Shape&, kvs_dtype, const void*, const void*, const int32_t*, const float*,
                        const float*, const float*, const uint8_t*, const int32_t*, void*, void*, int32_t*, hipStream_t) { check_table(tab); return ok(); }
hipError_t launch_merge_norms(const UnitTable& tab, const Shape&, kvs_dtype, const void*, const void*, const int32_t*, const float*,
                              const float*, const uint8_t*, const int32_t*, void*, void*, int32_t*, hipStream_t) { check_table(tab); return ok(); }
hipError_t launch_per_query_norms(const UnitTable& tab, const Shape&, const void*, const void*, const void*, const int32_t*,
                                  const float*, float*, uint16_t*, uint16_t*, float*, float*, float*, hipStream_t) { check_table(tab); return ok(); }
hipError_t launch_per_query_norms_f32(const UnitTable& tab, const Shape&, const void*, const void*, const void*, const int32_t*,
                                      const float*, float*, float*, float*, float*, hipStream_t) { check_table(tab); return ok(); }
hipError_t launch_decode(const UnitTable& tab, const Shape&, kvs_dtype, const void*, const void*, const void*, const int32_t*,
                         float*, float*, hipStream_t) { check_table(tab); return ok(); }

}  // namespace kvs
