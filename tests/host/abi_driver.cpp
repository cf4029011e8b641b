// Drives the host layer of libkvs (kvs_api.hip, linked with launch_stubs.cpp) through its C ABI on the CPU: argument
// errors, workspace sizing and carve-up, alias checks, and whole calls on problems of many ragged units whose
// "launches" are stubs.  Built with -fsanitize=address,undefined by tests/test_host_sanitizers.py: any out-of-bounds
// access, overflow or misaligned access in make_plan / carve / check_ranges / for_each_group ends the run.
// Device pointers are fake addresses that nothing dereferences.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "kvs.h"
#include "kvs_debug.h"

namespace kvs { int stub_launches(); }

static int g_failed = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED %s (line %d)\n", #cond, __LINE__); ++g_failed; } } while (0)

struct Problem {
  std::vector<int32_t> len, budget;
  std::vector<int64_t> in_row, out_row;
  kvs_problem p{};
  long long rows_in = 0, rows_out = 0;
  Problem(std::vector<int32_t> l, std::vector<int32_t> b, int group, int window, int D, kvs_dtype dt) : len(l), budget(b) {
    for (size_t i = 0; i < len.size(); ++i) {
      in_row.push_back(rows_in);
      out_row.push_back(rows_out);
      rows_in += len[i];
      rows_out += std::min(len[i], budget[i]);
    }
    p.n_units = (int)len.size(); p.group = group; p.window = window; p.head_dim = D; p.n_sink = 4; p.n_recent = 0;
    p.io_dtype = dt; p.scale = 0.f; p.len = len.data(); p.budget = budget.data(); p.in_row = in_row.data();
    p.out_row = out_row.data(); p.key_rule = KVS_RULE_HESSIAN; p.causal = 0;
  }
};

// fake, non-overlapping, 256-byte aligned device ranges
struct Arena {
  uintptr_t next = (uintptr_t)1 << 40;
  void* take(size_t bytes) { void* r = (void*)next; next += (bytes + 4095) / 4096 * 4096 + 4096; return r; }
};

static void whole_calls(std::mt19937& rng, kvs_dtype dt, int group, int window, int D) {
  const size_t elt = dt == KVS_F32 ? 4 : 2;
  for (int rep = 0; rep < 20; ++rep) {
    const int nu = 1 + (int)(rng() % 150);                      // up to three launch groups
    std::vector<int32_t> len(nu), budget(nu);
    for (int u = 0; u < nu; ++u) {
      len[u] = 32 + (int)(rng() % (rep % 4 == 0 ? 200000 : 9000));
      budget[u] = std::max(8, (int)(len[u] / (2 + rng() % 6)));
      if (rng() % 11 == 0) budget[u] = len[u] + 3;               // pass-through
    }
    Problem pr(len, budget, group, window, D, dt);
    const int R = group * window;
    size_t ws_bytes = 0, pq_bytes = 0, dec_bytes = 0;
    EXPECT(kvs_workspace_size(&pr.p, &ws_bytes) == KVS_OK);
    EXPECT(ws_bytes % 256 == 0 && ws_bytes >= (size_t)pr.rows_in * 9);
    Arena a;
    void* Q = a.take((size_t)nu * R * D * elt);
    void* K = a.take((size_t)pr.rows_in * D * elt);
    void* V = a.take((size_t)pr.rows_in * D * elt);
    void* Ko = a.take((size_t)pr.rows_out * D * elt);
    void* Vo = a.take((size_t)pr.rows_out * D * elt);
    int32_t* cnt = (int32_t*)a.take((size_t)pr.rows_out * 4);
    float* alpha = (float*)a.take((size_t)pr.rows_in * 4);
    float* obar = (float*)a.take((size_t)nu * D * 4);
    uint8_t* mask = (uint8_t*)a.take((size_t)pr.rows_in);
    int32_t* slot = (int32_t*)a.take((size_t)pr.rows_in * 4);
    int32_t* cin = (int32_t*)a.take((size_t)pr.rows_in * 4);
    void* ws = a.take(ws_bytes);
    const int before = kvs::stub_launches();
    EXPECT(kvs_step(&pr.p, Q, K, V, Ko, Vo, cnt, slot, mask, ws, ws_bytes, nullptr) == KVS_OK);
    EXPECT(kvs_step_counts(&pr.p, Q, K, V, cin, Ko, Vo, cnt, nullptr, nullptr, ws, ws_bytes, nullptr) == KVS_OK);
    EXPECT(kvs_score(&pr.p, Q, K, V, alpha, obar, ws, ws_bytes, nullptr) == KVS_OK);
    EXPECT(kvs_select(&pr.p, alpha, mask, slot, nullptr, 0, nullptr) == KVS_OK);
    EXPECT(kvs_select(&pr.p, alpha, mask, slot, ws, ws_bytes, nullptr) == KVS_OK);          // several workgroups per unit
    EXPECT(kvs_select(&pr.p, alpha, mask, slot, ws, ws_bytes - 256, nullptr) == KVS_OK);    // too small: not used
    EXPECT(kvs_select(&pr.p, alpha, (uint8_t*)ws, slot, ws, ws_bytes, nullptr) == KVS_ERR_ALIAS);
    EXPECT(kvs_merge_compact(&pr.p, K, V, alpha, obar, mask, slot, Ko, Vo, cnt, nullptr, 0, nullptr) == KVS_OK);
    EXPECT(kvs_merge_compact(&pr.p, K, V, alpha, obar, mask, slot, Ko, Vo, cnt, ws, ws_bytes, nullptr) == KVS_OK);   // optional
    EXPECT(kvs_merge_compact(&pr.p, K, V, alpha, obar, mask, slot, Ko, Vo, cnt, ws, ws_bytes - 256, nullptr) == KVS_OK);
    EXPECT(kvs_merge_compact(&pr.p, K, V, alpha, obar, (uint8_t*)ws, slot, Ko, Vo, cnt, ws, ws_bytes, nullptr) == KVS_ERR_ALIAS);
    EXPECT(kvs::stub_launches() >= before + 5 * ((nu + 63) / 64));
    EXPECT(kvs_step(&pr.p, Q, K, V, Ko, Vo, cnt, slot, mask, ws, ws_bytes - 1, nullptr) == KVS_ERR_WORKSPACE);
    EXPECT(kvs_step(&pr.p, Q, K, V, Ko, Ko, cnt, slot, mask, ws, ws_bytes, nullptr) == KVS_ERR_ALIAS);
    EXPECT(kvs_step(&pr.p, Q, K, V, Ko, Vo, cnt, slot, (uint8_t*)ws + 256, ws, ws_bytes, nullptr) == KVS_ERR_ALIAS);
    {                                          // per-query aggregation: both dtypes
      EXPECT(kvs_per_query_workspace_size(&pr.p, &pq_bytes) == KVS_OK && pq_bytes > ws_bytes);
      void* pws = a.take(pq_bytes);
      float* a_tok = (float*)a.take((size_t)pr.rows_in * 4);
      float* c_edge = (float*)a.take((size_t)pr.rows_in * 4);
      EXPECT(kvs_sensitivity(&pr.p, Q, K, V, alpha, a_tok, c_edge, pws, pq_bytes, nullptr) == KVS_OK);
      EXPECT(kvs_step_per_query(&pr.p, Q, K, V, Ko, Vo, cnt, nullptr, nullptr, pws, pq_bytes, nullptr) == KVS_OK);
      EXPECT(kvs_merge_compact_norms(&pr.p, K, V, a_tok, c_edge, mask, slot, Ko, Vo, cnt, nullptr, 0, nullptr) == KVS_OK);
      EXPECT(kvs_merge_compact_norms(&pr.p, K, V, a_tok, c_edge, mask, slot, Ko, Vo, cnt, ws, ws_bytes, nullptr) == KVS_OK);
      EXPECT(kvs_sensitivity_counts(&pr.p, Q, K, V, cin, alpha, a_tok, c_edge, pws, pq_bytes, nullptr) == KVS_OK);
      EXPECT(kvs_step_per_query_counts(&pr.p, Q, K, V, cin, Ko, Vo, cnt, nullptr, nullptr, pws, pq_bytes, nullptr) == KVS_OK);
      EXPECT(kvs_merge_compact_norms_counts(&pr.p, K, V, cin, a_tok, c_edge, mask, slot, Ko, Vo, cnt, nullptr, 0, nullptr) == KVS_OK);
      EXPECT(kvs_sensitivity_counts(&pr.p, Q, K, V, (const int32_t*)a_tok, alpha, a_tok, c_edge, pws, pq_bytes, nullptr) == KVS_ERR_ALIAS);
    }
    if (R <= KVS_MAX_DECODE_ROWS) {
      EXPECT(kvs_decode_workspace_size(&pr.p, &dec_bytes) == KVS_OK);
      float* out = (float*)a.take((size_t)nu * R * D * 4);
      void* dws = a.take(dec_bytes);
      EXPECT(kvs_decode_attention(&pr.p, Q, K, V, cin, out, dws, dec_bytes, nullptr) == KVS_OK);
    }
    // the static entry refuses what its array cannot hold, before any device call
    if (ws_bytes > KVS_STATIC_SCRATCH_BYTES) {
      EXPECT(kvs_step_static(&pr.p, Q, K, V, nullptr, Ko, Vo, cnt, nullptr, nullptr, nullptr) == KVS_ERR_WORKSPACE);
    }
  }
}

int main() {
  std::mt19937 rng(12345);
  size_t bytes = 0;
  EXPECT(kvs_workspace_size(nullptr, &bytes) == KVS_ERR_INVALID_ARG);
  {
    Problem pr({1024, 500}, {512, 600}, 2, 4, 64, KVS_F32);
    EXPECT(kvs_workspace_size(&pr.p, nullptr) == KVS_ERR_INVALID_ARG);
    EXPECT(kvs_workspace_size(&pr.p, &bytes) == KVS_OK && bytes % 256 == 0);
    kvs_problem q = pr.p;
    q.head_dim = 96; EXPECT(kvs_workspace_size(&q, &bytes) == KVS_ERR_INVALID_ARG);
    q = pr.p; q.group = 64; q.window = 32; EXPECT(kvs_workspace_size(&q, &bytes) == KVS_ERR_INVALID_ARG);
    q = pr.p; q.io_dtype = (kvs_dtype)7; EXPECT(kvs_workspace_size(&q, &bytes) == KVS_ERR_DTYPE);
    q = pr.p; q.len = nullptr; EXPECT(kvs_workspace_size(&q, &bytes) == KVS_ERR_INVALID_ARG);
    q = pr.p; q.n_units = 0; EXPECT(kvs_workspace_size(&q, &bytes) == KVS_ERR_INVALID_ARG);
    q = pr.p; q.causal = 2; EXPECT(kvs_workspace_size(&q, &bytes) == KVS_ERR_INVALID_ARG);
    q = pr.p; q.key_rule = (kvs_key_rule)5; EXPECT(kvs_workspace_size(&q, &bytes) == KVS_ERR_INVALID_ARG);
  }
  {
    Problem pr({KVS_MAX_LEN, 5}, {KVS_MAX_LEN / 2, 5}, 4, 32, 128, KVS_BF16);       // the longest unit, 32-bit offsets
    EXPECT(kvs_workspace_size(&pr.p, &bytes) == KVS_OK);
    Problem bad({KVS_MAX_LEN + 1, 5}, {KVS_MAX_LEN / 2, 5}, 4, 32, 128, KVS_BF16);
    EXPECT(kvs_workspace_size(&bad.p, &bytes) == KVS_ERR_INVALID_ARG);
    Problem small({1024, 500}, {3, 600}, 2, 4, 64, KVS_F32);                        // budget below n_sink + 1
    EXPECT(kvs_workspace_size(&small.p, &bytes) == KVS_ERR_BUDGET);
    Problem overlap({1024, 500}, {512, 600}, 2, 4, 64, KVS_F32);
    overlap.in_row[1] = 1000;
    EXPECT(kvs_workspace_size(&overlap.p, &bytes) == KVS_ERR_INVALID_ARG);
  }
  whole_calls(rng, KVS_F32, 1, 8, 64);
  whole_calls(rng, KVS_BF16, 4, 32, 128);       // the one-pass score kernel's tables are part of the workspace
  whole_calls(rng, KVS_BF16, 8, 64, 128);       // 512 query rows
  whole_calls(rng, KVS_BF16, 1, 3, 64);
  kvs_debug_set(KVS_DEBUG_SCORE_FUSED, 2);
  whole_calls(rng, KVS_BF16, 4, 32, 128);
  kvs_debug_set(KVS_DEBUG_SCORE_FUSED, 0);
  kvs_debug_set(KVS_DEBUG_SELECT_SPLIT, 2);     // as many select workgroups per unit as the units can have
  whole_calls(rng, KVS_BF16, 4, 32, 128);
  kvs_debug_set(KVS_DEBUG_SELECT_SPLIT, 1);     // never more than one
  whole_calls(rng, KVS_F32, 1, 8, 64);
  kvs_debug_set(KVS_DEBUG_SELECT_SPLIT, 0);
  for (int cap : {7, 64, 100}) {                // launch groups held to a few units, to the inline descriptors, beyond them
    kvs_debug_set(KVS_DEBUG_GROUP_UNITS, cap);
    whole_calls(rng, KVS_BF16, 4, 32, 128);
  }
  kvs_debug_set(KVS_DEBUG_GROUP_UNITS, 0);
  EXPECT(kvs_debug_set(99, 1) == -1);
  std::printf(g_failed ? "host layer: %d checks failed\n" : "host layer: all checks passed (%d stub launches)\n",
              g_failed ? g_failed : kvs::stub_launches());
  return g_failed ? 1 : 0;
}
