// Select kernel (which adjacent pairs merge, and the slot of every token) and the o_bar pass,
// in ONE launch: both need nothing but alpha_bar, so the few select workgroups (one per unit,
// latency-bound) run beside the many streaming workgroups that read V once for
// o_bar = sum_t alpha_bar[t] V[t] (Sec. 4.1, Eq. attn_def_vec, with the window's mean distribution).
//
// Select, per unit: edge score sigma[m] = alpha_bar[m] + alpha_bar[m+1] for the eligible edges
// n_sink <= m <= len-2-n_recent (App. C, paragraph (i): pairs with small accumulated attention
// mass; Sec. 5: the first tokens are always preserved); the r = len - budget smallest scores are
// selected in one parallel step (Sec. 3.1), ties going to the lower index; consecutive selected
// edges chain into one output slot.  One workgroup of 1024 threads per unit.  Scores are
// non-negative floats, so their bit patterns order like unsigned integers: an MSB-first radix
// select (11 + 11 + 10 bits, LDS histograms; the keys stretched to their full span first, the
// digits after the first settled on a short list) finds the r-th smallest key T and how many
// keys equal to T are still wanted; a final pass in index order takes every key below T and the
// first `want` keys equal to T, and turns the selection into the slot map with DPP prefix scans
// and a scan over the 16 wavefronts.  Keys of units up to kLdsKeys edges are kept in LDS between
// the passes; longer units recompute them from alpha_bar (L2-resident) in every pass with the
// same stretched ranking.  In a launch of few units a long unit is selected by several workgroups
// ("parts") instead, which meet through an exchange area in device memory (see select_unit_split);
// the kernel exists in two LDS sizes (kLdsKeys and kLdsKeysSmall keys per workgroup).
//
// o_bar pass, per chunk of a unit: rows of V are read by LPR adjacent lanes (16 bytes each), scaled
// by alpha_bar[t] and summed per lane, then over the workgroup; the chunk's sum goes to the
// workspace; whoever needs o_bar (every merge workgroup, or a tiny reduce kernel when o_bar itself
// is an output) adds the chunks up in chunk order, so the result does not depend on timing and no
// device-wide fence is needed (one costs a whole L2 write-back on this chip).
#include "kvs_device.h"

namespace kvs {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kLdsKeys = kSelUnitKeys;    // keys a workgroup can keep in LDS: the full-size kernel ...
constexpr int kLdsKeysSmall = kSelPartKeys;   // ... and the one for launches whose units are short or split into parts
constexpr int kBins = 2048;

__device__ __forceinline__ uint32_t edge_key(const float* __restrict__ a, int m) {
  return __float_as_uint(a[m] + a[m + 1]);
}

__device__ __forceinline__ int lanes_below(uint64_t ballot, int lane) {
  return __popcll(ballot & ((1ull << lane) - 1ull));
}

constexpr int kCand = 2048;               // keys of the first-pass bin that are refined in LDS

template <int KEYS>
struct SelectSmemT {
  static constexpr int kKeys = KEYS;
  uint32_t keys[KEYS];
  uint32_t cand[kCand];
  int hist[kBins];
  int wave[kSelWaves];
  int pick[3];           // digit, keys below it, keys in it
  int lt[kSelWaves], eq[kSelWaves];
  uint32_t wmin[kSelWaves], wmax[kSelWaves];
  int ncand;
  int plt[kSelMaxParts], peq[kSelMaxParts];     // split selection: the parts' counts of selected keys
  uint8_t cpart[kCand];                         // ... and the part every listed key came from
};

// Inclusive prefix sum over the 64 lanes with DPP moves only (no LDS crossbar): four shifts inside
// every row of 16 lanes, then the last lane of row 0 / row 2 is broadcast into the next row, then
// lane 31 into the upper half.
__device__ __forceinline__ int wave_incl_scan(int x) {
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true);    // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true);    // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true);    // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true);    // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
  return x;
}

// Sum of x[w] over the wavefronts before wavefront `wave` (x: kSelWaves ints in LDS): lanes 0..15 take
// one entry each and scan them inside their DPP row.
__device__ __forceinline__ int waves_before(const int* x, int wave, int lane) {
  static_assert(kSelWaves == 16, "one DPP row");
  int v = lane < kSelWaves ? x[lane] : 0;
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);
  const int idx = __builtin_amdgcn_readfirstlane(wave);
  return idx ? __builtin_amdgcn_readlane(v, idx - 1) : 0;
}

// Exclusive scan of the histogram (two bins per thread); finds the bin that holds rank `want`
// (1-based), extends (prefix, pmask, want) by that digit and returns the number of keys in the bin.
template <typename SM>
__device__ __forceinline__ int pick_bin(SM& sm, int shift, int bins, uint32_t& prefix, uint32_t& pmask,
                                        int& want) {
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int h0 = sm.hist[2 * tid], h1 = sm.hist[2 * tid + 1];
  const int incl = wave_incl_scan(h0 + h1);
  if (lane == kWave - 1) sm.wave[wave] = incl;
  __syncthreads();
  const int base = waves_before(sm.wave, wave, lane);
  const int excl = base + incl - (h0 + h1);
  if (want > excl && want <= excl + h0) { sm.pick[0] = 2 * tid; sm.pick[1] = excl; sm.pick[2] = h0; }
  else if (want > excl + h0 && want <= excl + h0 + h1) { sm.pick[0] = 2 * tid + 1; sm.pick[1] = excl + h0; sm.pick[2] = h1; }
  __syncthreads();
  prefix |= (uint32_t)sm.pick[0] << shift;
  pmask |= (uint32_t)(bins - 1) << shift;
  want -= sm.pick[1];
  const int in_bin = sm.pick[2];
  __syncthreads();
  return in_bin;
}

// Minimum / maximum over the 64 lanes (same DPP walk as the scan; lane 63 ends up with the result).
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) {
  const int id = -1;
  x = min(x, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)x, 0x111, 0xF, 0xF, false));
  x = min(x, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)x, 0x112, 0xF, 0xF, false));
  x = min(x, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)x, 0x114, 0xF, 0xF, false));
  x = min(x, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)x, 0x118, 0xF, 0xF, false));
  x = min(x, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)x, 0x142, 0xA, 0xF, false));
  x = min(x, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)x, 0x143, 0xC, 0xF, false));
  return (uint32_t)__builtin_amdgcn_readlane((int)x, kWave - 1);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
  x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xF, 0xF, false));
  x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xF, 0xF, false));
  x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, false));
  x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xF, 0xF, false));
  x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xA, 0xF, false));
  x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xC, 0xF, false));
  return (uint32_t)__builtin_amdgcn_readlane((int)x, kWave - 1);
}

// The first digit of the threshold is known (prefix, pmask) and `want` is its rank among the keys that share
// it: settles the remaining 21 bits.  sm.cand[0 .. ncand) lists those keys when ncand <= kCand; otherwise the
// passes run over sm.keys[0 .. nkeys).  Returns the number of keys equal to the threshold; prefix is then the
// threshold and `want` the number of keys equal to it that are still wanted.
template <typename SM>
__device__ __forceinline__ int refine_threshold(SM& sm, const int ncand, const int nkeys, uint32_t& prefix,
                                                uint32_t& pmask, int& want) {
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  constexpr uint32_t kNone = 0xffffffffu;
  int n_equal;                         // keys equal to the threshold
  if (ncand <= kWave) {
    // A handful of candidates: all against all.  Lane i of every wavefront holds candidate i, wavefront
    // w compares with candidates 4w..4w+3 (one LDS address per read: a broadcast), and the partial
    // counts meet in LDS.  Ties go by list position: equal keys are interchangeable here, only the
    // counts below and at the threshold matter.
    int* below = sm.hist;              // the histogram is idle now
    int* same = sm.hist + kWave;
    int* before = sm.hist + 2 * kWave;
    if (tid < 3 * kWave) sm.hist[tid] = 0;
    __syncthreads();
    const uint32_t c = lane < ncand ? sm.cand[lane] : kNone;
    int b = 0, e = 0, f = 0;
#pragma unroll
    for (int jj = 0; jj < kWave / kSelWaves; ++jj) {
      const int j = wave * (kWave / kSelWaves) + jj;
      const uint32_t cj = j < ncand ? sm.cand[j] : kNone;
      b += cj < c;
      e += cj == c;
      f += (cj == c) & (j < lane);
    }
    if (lane < ncand) {
      if (b) atomicAdd(&below[lane], b);
      if (e) atomicAdd(&same[lane], e);
      if (f) atomicAdd(&before[lane], f);
    }
    __syncthreads();
    if (tid < ncand && below[tid] + before[tid] == want - 1) {
      sm.pick[0] = (int)c;
      sm.pick[1] = below[tid];
      sm.pick[2] = same[tid];
    }
    __syncthreads();
    prefix = (uint32_t)sm.pick[0];
    want -= sm.pick[1];
    n_equal = sm.pick[2];
  } else {
    const bool listed = (ncand <= kCand);
    const int shifts[2] = {10, 0};
    const int widths[2] = {11, 10};
    n_equal = 0;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int shift = shifts[pass];
      const int bins = 1 << widths[pass];
      for (int b = tid; b < kBins; b += kSelThreads) sm.hist[b] = 0;
      __syncthreads();
      if (listed) {
        for (int i = tid; i < ncand; i += kSelThreads) {
          const uint32_t k = sm.cand[i];
          if ((k & pmask) == prefix) atomicAdd(&sm.hist[(k >> shift) & (bins - 1)], 1);
        }
      } else {                            // a bin too crowded for the list: full passes over the keys
        for (int i = tid; i < nkeys; i += kSelThreads) {
          const uint32_t k = sm.keys[i];
          if ((k & pmask) == prefix) atomicAdd(&sm.hist[(k >> shift) & (bins - 1)], 1);
        }
      }
      __syncthreads();
      n_equal = pick_bin(sm, shift, bins, prefix, pmask, want);
    }
  }
  return n_equal;
}

// Select for a unit whose keys fit the LDS.  Key i' belongs to the edge after token lo_al + i', where
// lo_al <= lo is the first token whose alpha_bar element sits on a 16-byte boundary: groups of four
// keys then coincide with aligned groups of four elements of alpha_bar, edge_mask and slot.  Keys
// of tokens outside [lo, hi] are 0xffffffff: no threshold reaches them.  One CU does all of this,
// so the instruction count per key is what matters: groups that lie wholly inside [lo, hi] (all but
// the first and the last) take paths without per-key checks.
template <typename SM>
__device__ __forceinline__ void select_unit_cached(const Unit& un, const float* __restrict__ a,
                                                   uint8_t* __restrict__ mk, int32_t* __restrict__ sl, SM& sm,
                                                   int lo, int hi, int r) {
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int n = un.len;
  const int pad0 = (int)((un.in_row + lo) & 3);
  const int lo_al = lo - pad0;
  const int G = (hi - lo_al + 4) / 4;              // groups of four keys, at most SM::kKeys / 4
  constexpr int GPT = SM::kKeys / 4 / kSelThreads; // groups per thread
  constexpr uint32_t kNone = 0xffffffffu;
  uint4* k4 = reinterpret_cast<uint4*>(sm.keys);

  // ---- keys and the histogram of their first digit: all of a thread's loads are in flight together
  for (int b = tid; b < kBins; b += kSelThreads) sm.hist[b] = 0;
  if (tid == 0) sm.ncand = 0;
  __syncthreads();
  {
    float4 v[GPT];
    float nx[GPT];
#pragma unroll
    for (int u = 0; u < GPT; ++u) {
      const int g = u * kSelThreads + tid;
      const int m0 = lo_al + 4 * g;                // may lie up to 3 tokens before the unit: still alpha_bar
      v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      nx[u] = 0.f;
      if (m0 >= lo && m0 + 3 <= hi) {              // hi <= n - 2: element m0 + 4 exists
        v[u] = *reinterpret_cast<const float4*>(a + m0);
        nx[u] = a[m0 + 4];
      } else if (g < G) {                          // first or last group: nothing is read past the unit's end
        v[u].x = a[min(m0, n - 1)];
        v[u].y = a[min(m0 + 1, n - 1)];
        v[u].z = a[min(m0 + 2, n - 1)];
        v[u].w = a[min(m0 + 3, n - 1)];
        nx[u] = a[min(m0 + 4, n - 1)];
      }
    }
    // raw keys, their minimum and maximum
    uint32_t k[GPT][4];
    uint32_t kmin = kNone, kmax = 0;
#pragma unroll
    for (int u = 0; u < GPT; ++u) {
      const int g = u * kSelThreads + tid;
      const int m0 = lo_al + 4 * g;
      k[u][0] = __float_as_uint(v[u].x + v[u].y);
      k[u][1] = __float_as_uint(v[u].y + v[u].z);
      k[u][2] = __float_as_uint(v[u].z + v[u].w);
      k[u][3] = __float_as_uint(v[u].w + nx[u]);
      if (m0 >= lo && m0 + 3 <= hi) {
        kmin = min(kmin, min(min(k[u][0], k[u][1]), min(k[u][2], k[u][3])));
        kmax = max(kmax, max(max(k[u][0], k[u][1]), max(k[u][2], k[u][3])));
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = (g < G) && (m0 + j >= lo) && (m0 + j <= hi);
          k[u][j] = ok ? k[u][j] : kNone;
          kmin = min(kmin, k[u][j]);
          kmax = max(kmax, ok ? k[u][j] : 0u);
        }
      }
    }
    kmin = wave_min_u32(kmin);
    kmax = wave_max_u32(kmax);
    if (lane == 0) { sm.wmin[wave] = kmin; sm.wmax[wave] = kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) { kmin = min(kmin, sm.wmin[w]); kmax = max(kmax, sm.wmax[w]); }
    // Keys are ranked as (key - kmin) << lshift, the span stretched to 31 bits: monotone, and the
    // first digit then separates neighbouring tokens' keys, which mostly share their top IEEE bits
    // (equal digits in one wavefront instruction serialise in the LDS atomics).  Bit 31 stays clear,
    // so the out-of-range marker shares no digit with a real key.
    const uint32_t span = kmax - kmin;             // < 2^31: the keys are bit patterns of non-negative floats
    const int lshift = span ? __clz(span) - 1 : 0;
#pragma unroll
    for (int u = 0; u < GPT; ++u) {
      const int g = u * kSelThreads + tid;
      const int m0 = lo_al + 4 * g;
      if (m0 >= lo && m0 + 3 <= hi) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          k[u][j] = (k[u][j] - kmin) << lshift;
          atomicAdd(&sm.hist[k[u][j] >> 21], 1);
        }
        k4[g] = make_uint4(k[u][0], k[u][1], k[u][2], k[u][3]);
      } else if (g < G) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (k[u][j] != kNone) {
            k[u][j] = (k[u][j] - kmin) << lshift;
            atomicAdd(&sm.hist[k[u][j] >> 21], 1);
          }
        }
        k4[g] = make_uint4(k[u][0], k[u][1], k[u][2], k[u][3]);
      }
    }
  }
  __syncthreads();
  uint32_t prefix = 0, pmask = 0;
  int want = r;                        // rank (1-based) among the keys that share `prefix`
  pick_bin(sm, 21, 2048, prefix, pmask, want);

  // ---- the keys of that bin go to a short list (one LDS atomic per wavefront: every lane counts its
  //      matches, a scan gives it its place); the remaining 21 bits are settled on the list
  {
    uint4 q[GPT];
    int c = 0;
#pragma unroll
    for (int u = 0; u < GPT; ++u) {
      const int g = u * kSelThreads + tid;
      q[u] = make_uint4(kNone, kNone, kNone, kNone);
      if (g < G) q[u] = k4[g];
      c += (((q[u].x ^ prefix) >> 21) == 0) + (((q[u].y ^ prefix) >> 21) == 0) + (((q[u].z ^ prefix) >> 21) == 0) +
           (((q[u].w ^ prefix) >> 21) == 0);
    }
    const int incl = wave_incl_scan(c);
    const int tot = __builtin_amdgcn_readlane(incl, kWave - 1);
    if (tot > 0) {                                 // wavefront-uniform
      int base = 0;
      if (lane == 0) base = atomicAdd(&sm.ncand, tot);
      int pos = __builtin_amdgcn_readfirstlane(base) + incl - c;
      if (c > 0) {
#pragma unroll
        for (int u = 0; u < GPT; ++u) {
          const uint32_t kk[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (((kk[j] ^ prefix) >> 21) == 0) {
              if (pos < kCand) sm.cand[pos] = kk[j];
              ++pos;
            }
          }
        }
      }
    }
  }
  __syncthreads();
  const int n_equal = refine_threshold(sm, sm.ncand, 4 * G, prefix, pmask, want);   // keys equal to the threshold
  const uint32_t T = prefix;           // `want` keys equal to T are taken, the lowest indices first
  // When every key equal to T is taken (nearly always: T is then the only one), "selected" is simply
  // "below T + 1" and nothing has to be ranked.
  const bool simple = (n_equal == want);
  const uint32_t Tc = simple ? T + 1 : T;

  // ---- ordered pass: wavefront w owns the groups [g0, g1), lane l the groups g0 + it * 64 + l
  constexpr int ITS = SM::kKeys / 4 / kSelWaves / kWave;     // rounds per wavefront
  const int per_g = ((G + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
  const int g0 = min(G, wave * per_g), g1 = min(G, g0 + per_g);
  uint4 q[ITS];
  int n_lt = 0, n_eq = 0;               // wavefront totals: keys below Tc, keys equal to T (if they matter)
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    const int g = g0 + it * kWave + lane;
    q[it] = make_uint4(kNone, kNone, kNone, kNone);
    if (g < g1) q[it] = k4[g];
    n_lt += __popcll(__ballot(q[it].x < Tc)) + __popcll(__ballot(q[it].y < Tc)) + __popcll(__ballot(q[it].z < Tc)) +
            __popcll(__ballot(q[it].w < Tc));
  }
  if (!simple) {
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
      n_eq += __popcll(__ballot(q[it].x == T)) + __popcll(__ballot(q[it].y == T)) + __popcll(__ballot(q[it].z == T)) +
              __popcll(__ballot(q[it].w == T));
    }
  }
  if (lane == 0) { sm.lt[wave] = n_lt; sm.eq[wave] = n_eq; }
  __syncthreads();
  int eq_before = 0, sel_before = waves_before(sm.lt, wave, lane);
  if (!simple) {
    for (int w = 0; w < wave; ++w) {
      const int e = sm.eq[w];
      sel_before += min(max(want - eq_before, 0), e);
      eq_before += e;
    }
  }

  // Four tokens' mask bytes and slots; whole groups inside [lo, hi] go out as one 4-byte and one
  // 16-byte store.  `below`: selected edges before the group's first token.
  auto write_group = [&](int g, const bool* sel, int below) {
    const int m0 = lo_al + 4 * g;
    int s4[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { s4[j] = m0 + j - below; below += sel[j]; }
    if (m0 >= lo && m0 + 3 <= hi) {
      *reinterpret_cast<uint32_t*>(mk + m0) =
          (uint32_t)sel[0] | ((uint32_t)sel[1] << 8) | ((uint32_t)sel[2] << 16) | ((uint32_t)sel[3] << 24);
      *reinterpret_cast<int4*>(sl + m0) = make_int4(s4[0], s4[1], s4[2], s4[3]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (m0 + j >= lo && m0 + j <= hi) { mk[m0 + j] = sel[j] ? 1 : 0; sl[m0 + j] = s4[j]; }
      }
    }
  };

  if (n_eq == 0) {
    // nothing to rank in this wavefront (the usual case): all rounds' scans at once
    int cnt[ITS], incl[ITS];
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
      cnt[it] = (q[it].x < Tc) + (q[it].y < Tc) + (q[it].z < Tc) + (q[it].w < Tc);
      incl[it] = wave_incl_scan(cnt[it]);
    }
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
      const int g = g0 + it * kWave + lane;
      const bool sel[4] = {q[it].x < Tc, q[it].y < Tc, q[it].z < Tc, q[it].w < Tc};
      if (g < g1) write_group(g, sel, sel_before + incl[it] - cnt[it]);
      sel_before += __builtin_amdgcn_readlane(incl[it], kWave - 1);
    }
  } else {
    // ties with the threshold: ranked in index order, round by round
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
      const int g = g0 + it * kWave + lane;
      const uint32_t kk[4] = {q[it].x, q[it].y, q[it].z, q[it].w};
      bool sel[4], eq[4];
      int lane_eq = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        sel[j] = kk[j] < T;
        eq[j] = kk[j] == T;
        lane_eq += eq[j];
      }
      const int incl_eq = wave_incl_scan(lane_eq);
      int rank = eq_before + incl_eq - lane_eq;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (eq[j]) { sel[j] = rank < want; ++rank; }
      }
      eq_before += __builtin_amdgcn_readlane(incl_eq, kWave - 1);
      const int lane_cnt = sel[0] + sel[1] + sel[2] + sel[3];
      const int incl = wave_incl_scan(lane_cnt);
      if (g < g1) write_group(g, sel, sel_before + incl - lane_cnt);
      sel_before += __builtin_amdgcn_readlane(incl, kWave - 1);
    }
  }
  // tokens outside the eligible edge range
  for (int t = tid; t < lo && t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t; }
  for (int t = hi + 1 + tid; t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t - r; }
}

// Select for a unit whose keys do not fit the LDS: the passes of the radix select and the ordered pass read
// alpha_bar again each time.  Same key layout as select_unit_cached (groups of four edges on 16-byte boundaries
// of alpha_bar, 0xffffffff outside [lo, hi]), same ranking (stretched keys), same tie rule (lowest index first).
template <typename SM>
__device__ __forceinline__ void select_unit_long(const Unit& un, const float* __restrict__ a, uint8_t* __restrict__ mk,
                                                 int32_t* __restrict__ sl, SM& sm, int lo, int hi, int r) {
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int n = un.len;
  const int pad0 = (int)((un.in_row + lo) & 3);
  const int lo_al = lo - pad0;
  const int G = (hi - lo_al + 4) / 4;              // groups of four keys
  constexpr uint32_t kNone = 0xffffffffu;
  constexpr int UN = 4;                            // groups a lane fetches before it uses the first

  // raw keys (IEEE bit patterns) of group g; positions outside [lo, hi] and groups past the end hold kNone
  auto load4 = [&](int g, uint32_t (&k)[4]) {
    const int m0 = lo_al + 4 * g;                  // may lie up to 3 tokens before the unit: still alpha_bar
    if (m0 >= lo && m0 + 3 <= hi) {                // hi <= n - 2: element m0 + 4 exists
      const float4 v = *reinterpret_cast<const float4*>(a + m0);
      const float nx = a[m0 + 4];
      k[0] = __float_as_uint(v.x + v.y);
      k[1] = __float_as_uint(v.y + v.z);
      k[2] = __float_as_uint(v.z + v.w);
      k[3] = __float_as_uint(v.w + nx);
    } else if (g < G) {                            // first or last group: nothing is read past the unit's end
      float e[5];
#pragma unroll
      for (int j = 0; j < 5; ++j) e[j] = a[min(m0 + j, n - 1)];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = (m0 + j >= lo) && (m0 + j <= hi);
        k[j] = ok ? __float_as_uint(e[j] + e[j + 1]) : kNone;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) k[j] = kNone;
    }
  };
  // f(k[4]) for every group, any order; UN groups of a lane are in flight together
  auto for_groups = [&](auto&& f) {
    for (int base = 0; base < G; base += kSelThreads * UN) {
      uint32_t k[UN][4];
#pragma unroll
      for (int u = 0; u < UN; ++u) load4(base + u * kSelThreads + tid, k[u]);
#pragma unroll
      for (int u = 0; u < UN; ++u) f(k[u]);
    }
  };

  // ---- minimum and maximum: keys are ranked as (key - kmin) << lshift (monotone, bit 31 clear, and the first digit
  //      tells neighbouring tokens apart, whose raw keys share their top bits and would serialise the LDS atomics)
  uint32_t kmin = kNone, kmax = 0;
  for_groups([&](const uint32_t (&k)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      kmin = min(kmin, k[j]);
      kmax = max(kmax, k[j] == kNone ? 0u : k[j]);
    }
  });
  kmin = wave_min_u32(kmin);
  kmax = wave_max_u32(kmax);
  if (lane == 0) { sm.wmin[wave] = kmin; sm.wmax[wave] = kmax; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) { kmin = min(kmin, sm.wmin[w]); kmax = max(kmax, sm.wmax[w]); }
  const uint32_t span = kmax - kmin;               // < 2^31: the keys are bit patterns of non-negative floats
  const int lshift = span ? __clz(span) - 1 : 0;
  auto ranked = [&](uint32_t k) { return k == kNone ? kNone : (k - kmin) << lshift; };

  // ---- MSB-first radix select, 11 + 11 + 10 bits, every pass over all keys
  uint32_t prefix = 0, pmask = 0;
  int want = r;                        // rank (1-based) among the keys that share `prefix`
  int n_equal = 0;
  const int shifts[3] = {21, 10, 0};
  const int widths[3] = {11, 11, 10};
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = shifts[pass];
    const int bins = 1 << widths[pass];
    for (int b = tid; b < kBins; b += kSelThreads) sm.hist[b] = 0;
    __syncthreads();
    for_groups([&](const uint32_t (&k)[4]) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t q = ranked(k[j]);
        if (q != kNone && (q & pmask) == prefix) atomicAdd(&sm.hist[(q >> shift) & (bins - 1)], 1);
      }
    });
    __syncthreads();
    n_equal = pick_bin(sm, shift, bins, prefix, pmask, want);
  }
  const uint32_t T = prefix;           // `want` keys equal to T are taken, the lowest indices first
  const bool simple = (n_equal == want);          // every key equal to T is taken: "selected" is "below T + 1"
  const uint32_t Tc = simple ? T + 1 : T;

  // ---- ordered pass: wavefront w owns the groups [g0, g1), lane l the groups g0 + it * 64 + l
  const int per_g = ((G + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
  const int g0 = min(G, wave * per_g), g1 = min(G, g0 + per_g);
  int n_lt = 0, n_eq = 0;               // wavefront totals: keys below Tc, keys equal to T (if they matter)
  for (int gb = g0; gb < g1; gb += kWave * UN) {
    uint32_t k[UN][4];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int g = gb + u * kWave + lane;
      load4(g < g1 ? g : G, k[u]);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t q = ranked(k[u][j]);
        n_lt += __popcll(__ballot(q < Tc));
        if (!simple) n_eq += __popcll(__ballot(q == T));
      }
    }
  }
  if (lane == 0) { sm.lt[wave] = n_lt; sm.eq[wave] = n_eq; }
  __syncthreads();
  int eq_before = 0, sel_before = waves_before(sm.lt, wave, lane);
  if (!simple) {
    for (int w = 0; w < wave; ++w) {
      const int e = sm.eq[w];
      sel_before += min(max(want - eq_before, 0), e);
      eq_before += e;
    }
  }
  // Four tokens' mask bytes and slots; whole groups inside [lo, hi] go out as one 4-byte and one 16-byte store.
  // `below`: selected edges before the group's first token.
  auto write_group = [&](int g, const bool* sel, int below) {
    const int m0 = lo_al + 4 * g;
    int s4[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { s4[j] = m0 + j - below; below += sel[j]; }
    if (m0 >= lo && m0 + 3 <= hi) {
      *reinterpret_cast<uint32_t*>(mk + m0) =
          (uint32_t)sel[0] | ((uint32_t)sel[1] << 8) | ((uint32_t)sel[2] << 16) | ((uint32_t)sel[3] << 24);
      *reinterpret_cast<int4*>(sl + m0) = make_int4(s4[0], s4[1], s4[2], s4[3]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (m0 + j >= lo && m0 + j <= hi) { mk[m0 + j] = sel[j] ? 1 : 0; sl[m0 + j] = s4[j]; }
      }
    }
  };
  const bool ties = !simple && n_eq > 0;           // wavefront-uniform: keys equal to T must be ranked by index
  for (int gb = g0; gb < g1; gb += kWave * UN) {
    uint32_t k[UN][4];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int g = gb + u * kWave + lane;
      load4(g < g1 ? g : G, k[u]);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int g = gb + u * kWave + lane;
      bool sel[4];
      if (!ties) {
#pragma unroll
        for (int j = 0; j < 4; ++j) sel[j] = ranked(k[u][j]) < Tc;
      } else {
        bool eq[4];
        int lane_eq = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t q = ranked(k[u][j]);
          sel[j] = q < T;
          eq[j] = q == T;
          lane_eq += eq[j];
        }
        const int incl_eq = wave_incl_scan(lane_eq);
        int rank = eq_before + incl_eq - lane_eq;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (eq[j]) { sel[j] = rank < want; ++rank; }
        }
        eq_before += __builtin_amdgcn_readlane(incl_eq, kWave - 1);
      }
      const int lane_cnt = sel[0] + sel[1] + sel[2] + sel[3];
      const int incl = wave_incl_scan(lane_cnt);
      if (g < g1) write_group(g, sel, sel_before + incl - lane_cnt);
      sel_before += __builtin_amdgcn_readlane(incl, kWave - 1);
    }
  }
  // tokens outside the eligible edge range
  for (int t = tid; t < lo && t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t; }
  for (int t = hi + 1 + tid; t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t - r; }
}

// ---- selection of one unit by several workgroups ("parts") -----------------------------------------------------
// Every part owns a contiguous range of the unit's key groups and keeps its keys in LDS.  The parts meet three times
// through the unit's exchange area in device memory (zero at kernel start): smallest and largest key; histogram of
// the first digit; the keys of the threshold's bin, each with the part it came from, and every part's number of
// keys in the bins below.  From that list every part settles the same threshold and knows how many selected edges
// lie before its range, so nothing more has to be exchanged.  What crosses workgroups moves by agent-scope atomics,
// loads and stores, which pass the per-XCD L2 caches; a part bumps a phase's counter only after its own stores have
// completed.  The integer sums do not depend on the order in which the parts arrive, so the result is the
// single-workgroup one bit for bit.
// Every wait is bounded (clock and poll count).  A phase either completes for all parts or fails for all of them:
// its counter completes when it reads exactly P, and a part that runs out of time marks the counter with a
// compare-and-swap that only succeeds while the count is still short; after that it can never read exactly P again.
// When a phase fails every part leaves and the unit's first part selects the whole unit by itself.
constexpr unsigned kSelMaxPolls = 1u << 16;    // second bound on a wait, should the clock ever misbehave

__device__ __forceinline__ unsigned ld_agent(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(unsigned* p, unsigned v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned add_agent(unsigned* p, unsigned v) {
  return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool cas_agent(unsigned* p, unsigned expected, unsigned desired) {
  return __hip_atomic_compare_exchange_strong(p, &expected, desired, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void max_agent(unsigned* p, unsigned v) {
  (void)__hip_atomic_fetch_max(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_all_memory_ops() {
  __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0): this lane's loads, stores and atomics have completed
  asm volatile("" ::: "memory");
}

// This part has finished `phase`: all its threads' exchange-area writes are complete before the counter moves.
__device__ __forceinline__ void split_arrive(unsigned* g, int phase) {
  wait_all_memory_ops();
  __syncthreads();
  if (threadIdx.x == 0) (void)add_agent(&g[kSelArrive + phase], 1u);
}
// True once all P parts have finished `phase`; false when a part has run out of time there.  The answer is the same
// in every thread, and the same in every part.
template <typename SM>
__device__ __forceinline__ bool split_wait(unsigned* g, int phase, int P, unsigned timeout_ticks, SM& sm) {
  if (threadIdx.x == 0) {
    unsigned* word = &g[kSelArrive + phase];
    int ok = 0;
    const unsigned long long t_start = wall_clock64();
    for (unsigned poll = 0; poll < kSelMaxPolls; ++poll) {
      const unsigned v = ld_agent(word);
      if (v == (unsigned)P) { ok = 1; break; }
      if (v & kSelGaveUp) break;
      if (poll + 1 == kSelMaxPolls || wall_clock64() - t_start >= (unsigned long long)timeout_ticks) {
        // out of time: give up, unless the count has completed in the meantime (then the swap fails and the
        // next look at the counter sees it complete)
        if (cas_agent(word, v, v | kSelGaveUp)) break;
        if (poll + 1 == kSelMaxPolls) poll -= 1;     // (the value has changed at most P + 1 times: this ends)
        continue;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    sm.pick[0] = ok;
  }
  __syncthreads();
  const bool ok = sm.pick[0] != 0;
  __syncthreads();
  return ok;
}

// (-DKVS_SELECT_PROFILE: part 0 leaves the clock at the end of every phase in spare words of the exchange area)
#ifdef KVS_SELECT_PROFILE
#define SEL_STAMP(i) do { if (part == 0 && threadIdx.x == 0) st_agent(&g[48 + (i)], (unsigned)wall_clock64()); } while (0)
#else
#define SEL_STAMP(i) do { } while (0)
#endif

// Returns true when the unit's selection is complete; false when the parts could not finish together (part 0 then
// does the whole unit alone, the other parts have nothing left to do).
template <typename SM>
__device__ __forceinline__ bool select_unit_split(const Unit& un, const float* __restrict__ a, uint8_t* __restrict__ mk,
                                                  int32_t* __restrict__ sl, SM& sm, unsigned* g, const int part,
                                                  const int P, const int lo, const int hi, const int r,
                                                  const unsigned timeout_ticks) {
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int n = un.len;
  const int pad0 = (int)((un.in_row + lo) & 3);
  const int lo_al = lo - pad0;
  const int G = (hi - lo_al + 4) / 4;              // groups of four keys of the whole unit
  const int gpp = (G + P - 1) / P;                 // groups per part: at most kSelPartKeys / 4 (the host has seen to it)
  const int gp0 = min(G, part * gpp), gp1 = min(G, gp0 + gpp);
  const int GL = gp1 - gp0;                        // this part's groups; local group lg is group gp0 + lg of the unit
  constexpr int GPT = kSelPartKeys / 4 / kSelThreads;
  constexpr uint32_t kNone = 0xffffffffu;
  uint4* k4 = reinterpret_cast<uint4*>(sm.keys);

  SEL_STAMP(0);
  for (int b = tid; b < kBins; b += kSelThreads) sm.hist[b] = 0;
  if (tid == 0) sm.ncand = 0;

  // ---- phase 0: raw keys of this part, their minimum and maximum
  uint32_t k[GPT][4];
  uint32_t kmin = kNone, kmax = 0;
#pragma unroll
  for (int u = 0; u < GPT; ++u) {
    const int lg = u * kSelThreads + tid;
    const int m0 = lo_al + 4 * (gp0 + lg);         // may lie up to 3 tokens before the unit: still alpha_bar
    if (lg < GL && m0 >= lo && m0 + 3 <= hi) {     // hi <= n - 2: element m0 + 4 exists
      const float4 v = *reinterpret_cast<const float4*>(a + m0);
      const float nx = a[m0 + 4];
      k[u][0] = __float_as_uint(v.x + v.y);
      k[u][1] = __float_as_uint(v.y + v.z);
      k[u][2] = __float_as_uint(v.z + v.w);
      k[u][3] = __float_as_uint(v.w + nx);
    } else if (lg < GL) {                          // the unit's first or last group: nothing is read past its end
      float e[5];
#pragma unroll
      for (int j = 0; j < 5; ++j) e[j] = a[min(m0 + j, n - 1)];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = (m0 + j >= lo) && (m0 + j <= hi);
        k[u][j] = ok ? __float_as_uint(e[j] + e[j + 1]) : kNone;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) k[u][j] = kNone;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      kmin = min(kmin, k[u][j]);
      kmax = max(kmax, k[u][j] == kNone ? 0u : k[u][j]);
    }
  }
  kmin = wave_min_u32(kmin);
  kmax = wave_max_u32(kmax);
  if (lane == 0) { sm.wmin[wave] = kmin; sm.wmax[wave] = kmax; }
  __syncthreads();
  if (tid == 0) {
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) { kmin = min(kmin, sm.wmin[w]); kmax = max(kmax, sm.wmax[w]); }
    max_agent(&g[kSelNotMin], ~kmin);              // (the area starts from zero: the minimum travels complemented)
    max_agent(&g[kSelMax], kmax);
  }
  SEL_STAMP(1);
  split_arrive(g, 0);
  if (!split_wait(g, 0, P, timeout_ticks, sm)) return false;
  SEL_STAMP(2);
  kmin = ~ld_agent(&g[kSelNotMin]);
  kmax = ld_agent(&g[kSelMax]);

  // ---- phase 1: keys ranked as in the single-workgroup selection ((key - kmin) << lshift), this part's histogram
  //      of the first digit added to the unit's
  const uint32_t span = kmax - kmin;
  const int lshift = span ? __clz(span) - 1 : 0;
#pragma unroll
  for (int u = 0; u < GPT; ++u) {
    const int lg = u * kSelThreads + tid;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (k[u][j] != kNone) {
        k[u][j] = (k[u][j] - kmin) << lshift;
        atomicAdd(&sm.hist[k[u][j] >> 21], 1);
      }
    }
    if (lg < GL) k4[lg] = make_uint4(k[u][0], k[u][1], k[u][2], k[u][3]);
  }
  __syncthreads();
  {
    const int h0 = sm.hist[2 * tid], h1 = sm.hist[2 * tid + 1];
    if (h0) (void)add_agent(&g[kSelHist + 2 * tid], (unsigned)h0);
    if (h1) (void)add_agent(&g[kSelHist + 2 * tid + 1], (unsigned)h1);
  }
  SEL_STAMP(3);
  split_arrive(g, 1);
  if (!split_wait(g, 1, P, timeout_ticks, sm)) return false;
  SEL_STAMP(4);
  sm.hist[2 * tid] = (int)ld_agent(&g[kSelHist + 2 * tid]);
  sm.hist[2 * tid + 1] = (int)ld_agent(&g[kSelHist + 2 * tid + 1]);
  __syncthreads();
  uint32_t prefix = 0, pmask = 0;
  int want = r;                        // rank (1-based) among the keys that share `prefix`
  const int nb = pick_bin(sm, 21, 2048, prefix, pmask, want);
  if (nb > kSelCandMax) return false;  // a bin too crowded for the list: every part sees that and leaves the same way

  // ---- phase 2: this part's keys of that bin -> the unit's list, each with the number of this part; and how many
  //      of this part's keys lie in the bins below
  const uint32_t bstar = prefix >> 21;
  {
    int c = 0, low = 0;
#pragma unroll
    for (int u = 0; u < GPT; ++u) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        c += (((k[u][j] ^ prefix) >> 21) == 0);
        low += ((k[u][j] >> 21) < bstar);          // (a position outside the eligible range has the top digit)
      }
    }
    const int incl = wave_incl_scan(c);
    const int tot = __builtin_amdgcn_readlane(incl, kWave - 1);
    const int low_w = __builtin_amdgcn_readlane(wave_incl_scan(low), kWave - 1);
    if (lane == 0) sm.lt[wave] = low_w;
    if (tot > 0) {                                 // wavefront-uniform
      int base = 0;
      if (lane == 0) base = atomicAdd(&sm.ncand, tot);
      int pos = __builtin_amdgcn_readfirstlane(base) + incl - c;
#pragma unroll
      for (int u = 0; u < GPT; ++u) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (((k[u][j] ^ prefix) >> 21) == 0) {
            if (pos < kCand) sm.cand[pos] = k[u][j];
            ++pos;
          }
        }
      }
    }
  }
  __syncthreads();
  const int mine = sm.ncand;                       // <= nb <= kSelCandMax
  if (tid == 0) {
    int low = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) low += sm.lt[w];
    st_agent(&g[kSelPartLow + part], (unsigned)low);
    sm.pick[1] = mine ? (int)add_agent(&g[kSelNCand], (unsigned)mine) : 0;
  }
  __syncthreads();
  const int gbase = sm.pick[1];
  for (int i = tid; i < mine; i += kSelThreads) {
    if (gbase + i < kSelCandMax) {
      st_agent(&g[kSelCand + gbase + i], sm.cand[i]);
      st_agent(&g[kSelCandPart + gbase + i], (unsigned)part);
    }
  }
  SEL_STAMP(5);
  split_arrive(g, 2);
  if (!split_wait(g, 2, P, timeout_ticks, sm)) return false;
  SEL_STAMP(6);
  for (int i = tid; i < nb; i += kSelThreads) {
    sm.cand[i] = ld_agent(&g[kSelCand + i]);
    sm.cpart[i] = (uint8_t)ld_agent(&g[kSelCandPart + i]);
  }
  if (tid < kSelMaxParts) {                        // the parts' keys below the threshold's bin
    sm.plt[tid] = tid < P ? (int)ld_agent(&g[kSelPartLow + tid]) : 0;
    sm.peq[tid] = 0;
  }
  __syncthreads();
  const int n_equal = refine_threshold(sm, nb, 0, prefix, pmask, want);
  const uint32_t T = prefix;           // `want` keys equal to T are taken, the lowest indices first
  const bool simple = (n_equal == want);
  const uint32_t Tc = simple ? T + 1 : T;
  // every part's keys of the threshold's bin that lie below Tc, and those equal to T when they have to be ranked
  for (int i = tid; i < nb; i += kSelThreads) {
    const uint32_t ck = sm.cand[i];
    const int cp = sm.cpart[i];
    if (ck < Tc) atomicAdd(&sm.plt[cp], 1);
    else if (!simple && ck == T) atomicAdd(&sm.peq[cp], 1);
  }
  // (the barrier after the wavefront counts below also covers these sums)

  // ---- ordered pass.  Wavefront w owns the local groups [g0, g1), lane l the groups g0 + it * 64 + l.
  constexpr int ITS = kSelPartKeys / 4 / kSelWaves / kWave;
  constexpr int per_g = ITS * kWave;
  const int g0 = min(GL, wave * per_g), g1 = min(GL, g0 + per_g);
  uint4 q[ITS];
  int n_lt = 0, n_eq = 0;               // wavefront totals: keys below Tc, keys equal to T (if they matter)
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    const int lg = g0 + it * kWave + lane;
    q[it] = make_uint4(kNone, kNone, kNone, kNone);
    if (lg < g1) q[it] = k4[lg];
    n_lt += __popcll(__ballot(q[it].x < Tc)) + __popcll(__ballot(q[it].y < Tc)) + __popcll(__ballot(q[it].z < Tc)) +
            __popcll(__ballot(q[it].w < Tc));
    if (!simple) {
      n_eq += __popcll(__ballot(q[it].x == T)) + __popcll(__ballot(q[it].y == T)) + __popcll(__ballot(q[it].z == T)) +
              __popcll(__ballot(q[it].w == T));
    }
  }
  if (lane == 0) { sm.lt[wave] = n_lt; sm.eq[wave] = n_eq; }
  __syncthreads();
  SEL_STAMP(7);
  int eq_before = 0, sel_before = 0;    // over the parts before this one, then the wavefronts before this one
  for (int p = 0; p < part; ++p) {
    sel_before += sm.plt[p];
    if (!simple) {
      const int e = sm.peq[p];
      sel_before += min(max(want - eq_before, 0), e);
      eq_before += e;
    }
  }
  sel_before += waves_before(sm.lt, wave, lane);
  if (!simple) {
    for (int w = 0; w < wave; ++w) {
      const int e = sm.eq[w];
      sel_before += min(max(want - eq_before, 0), e);
      eq_before += e;
    }
  }
  // Four tokens' mask bytes and slots; `below`: selected edges before the group's first token.
  auto write_group = [&](int gg, const bool* sel, int below) {
    const int m0 = lo_al + 4 * gg;
    int s4[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { s4[j] = m0 + j - below; below += sel[j]; }
    if (m0 >= lo && m0 + 3 <= hi) {
      *reinterpret_cast<uint32_t*>(mk + m0) =
          (uint32_t)sel[0] | ((uint32_t)sel[1] << 8) | ((uint32_t)sel[2] << 16) | ((uint32_t)sel[3] << 24);
      *reinterpret_cast<int4*>(sl + m0) = make_int4(s4[0], s4[1], s4[2], s4[3]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (m0 + j >= lo && m0 + j <= hi) { mk[m0 + j] = sel[j] ? 1 : 0; sl[m0 + j] = s4[j]; }
      }
    }
  };
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    const int lg = g0 + it * kWave + lane;
    const uint32_t kk[4] = {q[it].x, q[it].y, q[it].z, q[it].w};
    bool sel[4];
    if (n_eq == 0) {                               // wavefront-uniform: nothing to rank here
#pragma unroll
      for (int j = 0; j < 4; ++j) sel[j] = kk[j] < Tc;
    } else {                                       // ties with the threshold: ranked in index order
      bool eq[4];
      int lane_eq = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        sel[j] = kk[j] < T;
        eq[j] = kk[j] == T;
        lane_eq += eq[j];
      }
      const int incl_eq = wave_incl_scan(lane_eq);
      int rank = eq_before + incl_eq - lane_eq;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (eq[j]) { sel[j] = rank < want; ++rank; }
      }
      eq_before += __builtin_amdgcn_readlane(incl_eq, kWave - 1);
    }
    const int lane_cnt = sel[0] + sel[1] + sel[2] + sel[3];
    const int incl = wave_incl_scan(lane_cnt);
    if (lg < g1) write_group(gp0 + lg, sel, sel_before + incl - lane_cnt);
    sel_before += __builtin_amdgcn_readlane(incl, kWave - 1);
  }
  // tokens outside the eligible edge range
  if (part == 0) {
    for (int t = tid; t < lo && t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t; }
  }
  if (part == P - 1) {
    for (int t = hi + 1 + tid; t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t - r; }
  }
  SEL_STAMP(8);
  return true;
}

template <typename SM>
__device__ __forceinline__ void select_unit(const Unit& un, const Shape& sh, const float* __restrict__ alpha_bar,
                            uint8_t* __restrict__ edge_mask, int32_t* __restrict__ slot, SM& sm) {
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int n = un.len;
  const int r = n - un.n_out;
  const float* a = alpha_bar + un.in_row;
  uint8_t* mk = edge_mask + un.in_row;
  int32_t* sl = slot + un.in_row;

  const int lo = sh.n_sink;
  const int hi = n - 2 - sh.n_recent;
  const int E = hi - lo + 1;           // eligible edges; the host has checked r <= E whenever r > 0
  if (r <= 0 || E <= 0) {
    for (int t = tid; t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t; }
    return;
  }
  if (E + 6 <= SM::kKeys) {            // with the padding to aligned groups of four at both ends
    select_unit_cached(un, a, mk, sl, sm, lo, hi, r);
    return;
  }

  // ---- longer units: every pass recomputes the keys from alpha_bar (L2-resident).  One CU walks the whole unit
  //      several times, so the instruction count per key is what counts: as in the cached path a lane takes four
  //      consecutive edges from one aligned 16-byte load plus one element, whole groups inside [lo, hi] skip the
  //      per-key checks, keys are ranked stretched, and the ordered pass writes four tokens per lane.
  select_unit_long(un, a, mk, sl, sm, lo, hi, r);
}

template <typename T, int D, bool STREAM>
__device__ __forceinline__ void obar_chunk(const Unit& un, int chunk, const T* __restrict__ V,
                                           const int32_t* __restrict__ counts_in, const float* __restrict__ alpha_bar,
                                           float* __restrict__ o_part, float (*sm_o)[128]) {
  constexpr int EPL = Piece<T>::N;
  constexpr int LPR = D / EPL;
  constexpr int RPW = kWave / LPR;
  constexpr int RPB = RPW * kSelWaves;
  constexpr int UNROLL = 4;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int grp = lane / LPR, piece = lane % LPR;
  const int clen = obar_chunk_len(un.len);
  const int t0 = chunk * clen;
  const int t1 = min(un.len, t0 + clen);
  const uint4* Vp = reinterpret_cast<const uint4*>(V + (size_t)un.in_row * D) + piece;
  const float* al = alpha_bar + un.in_row;
  const int32_t* cnt = counts_in ? counts_in + un.in_row : nullptr;   // rows that are sums over c tokens: v = V / c

  float acc[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) acc[i] = 0.f;
  for (int tb = t0 + wave * RPW + grp; tb < t1; tb += RPB * UNROLL) {
    uint4 raw[UNROLL];
    float a[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int t = tb + u * RPB;
      const int tc = min(t, t1 - 1);
      {   // a launch larger than the caches reads V non-temporally: the stream then does not sweep L2
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        const u32x4* src = reinterpret_cast<const u32x4*>(Vp + (size_t)tc * LPR);
        const u32x4 r = STREAM ? __builtin_nontemporal_load(src) : *src;
        raw[u] = make_uint4(r.x, r.y, r.z, r.w);
      }
      a[u] = (t < t1) ? al[tc] : 0.f;
      if (cnt) a[u] = a[u] / (float)cnt[tc];
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      float vf[EPL];
      Piece<T>::unpack(raw[u], vf);
#pragma unroll
      for (int i = 0; i < EPL; ++i) acc[i] = fmaf(a[u], vf[i], acc[i]);
    }
  }
  // lanes that hold the same piece of the row, then the wavefronts, in a fixed order
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] += __shfl_xor(acc[i], off, kWave);
  }
  if (grp == 0) {
#pragma unroll
    for (int i = 0; i < EPL; ++i) sm_o[wave][piece * EPL + i] = acc[i];
  }
  __syncthreads();
  if (tid < D) {
    float s = 0.f;
    for (int w = 0; w < kSelWaves; ++w) s += sm_o[w][tid];
    o_part[((size_t)un.index * kMaxChunks + chunk) * D + tid] = s;
  }
}

// o_bar[unit] = the unit's partial sums added in chunk order (thread d takes channel d; UN loads in flight).
__device__ __forceinline__ void obar_reduce_unit(const Unit& un, const Shape& sh, const float* __restrict__ parts,
                                                 float* __restrict__ o_bar) {
  const int nc = obar_partials(sh, un);
  const float* src = parts + obar_partial_at(sh, un, 0);
  constexpr int UN = 8;
  for (int d = threadIdx.x; d < sh.D; d += blockDim.x) {
    float s = 0.f;
    for (int c0 = 0; c0 < nc; c0 += UN) {
      float v[UN];
#pragma unroll
      for (int u = 0; u < UN; ++u) v[u] = (c0 + u < nc) ? src[(size_t)(c0 + u) * sh.D + d] : 0.f;
#pragma unroll
      for (int u = 0; u < UN; ++u) s += v[u];
    }
    o_bar[(size_t)un.index * sh.D + d] = s;
  }
}

// Three kinds of workgroups: blocks [0, n_select) select one unit's edges each, blocks [n_select, n_select +
// n_reduce) add one unit's partial o_bar sums up each, the others stream one chunk of V each.
// KEYS: edge scores a select workgroup can keep in LDS.  The small size leaves room for three workgroups per CU,
// which matters to the workgroups of the other kinds in the same launch.
template <typename T, int D, int KEYS>
__global__ __launch_bounds__(kSelThreads) void select_obar_kernel(
    const UnitTable tab, const Shape sh, const int n_select, const int n_reduce, const float* __restrict__ alpha_bar,
    uint8_t* __restrict__ edge_mask, int32_t* __restrict__ slot, const T* __restrict__ V,
    const int32_t* __restrict__ counts_in, float* __restrict__ o_part, const float* __restrict__ parts_in,
    float* __restrict__ o_bar_out, unsigned int* sel_shared, const unsigned timeout_ticks) {
  __shared__ SelectSmemT<KEYS> sm;
  __shared__ float sm_o[kSelWaves][128];
  const int b = blockIdx.x;
  if (b < n_select) {
    const int ui = n_select == tab.n_units ? b : find_unit_by<&Unit::s_base>(tab, b);     // (one workgroup per unit: no search)
    const Unit un = tab.unit(ui);
    const int P = (ui + 1 < tab.n_units ? tab.unit(ui + 1).s_base : tab.total_sparts) - un.s_base;
    if (P <= 1) {
      select_unit(un, sh, alpha_bar, edge_mask, slot, sm);
    } else {
      // (the host gives a unit several parts only when it has edges to select: r > 0, lo <= hi)
      const int part = b - un.s_base;
      const bool done = select_unit_split(un, alpha_bar + un.in_row, edge_mask + un.in_row, slot + un.in_row, sm,
                                          sel_shared + (size_t)ui * kSelSharedInts, part, P, sh.n_sink,
                                          un.len - 2 - sh.n_recent, un.len - un.n_out, timeout_ticks);
      if (!done && part == 0) {
        __syncthreads();
        select_unit(un, sh, alpha_bar, edge_mask, slot, sm);
      }
    }
  } else if (b < n_select + n_reduce) {
    obar_reduce_unit(tab.unit(b - n_select), sh, parts_in, o_bar_out);
  } else {
    const int c = b - n_select - n_reduce;
    const int ui = find_unit_by<&Unit::o_base>(tab, c);
    if (sh.stream) obar_chunk<T, D, true>(tab.unit(ui), c - tab.unit(ui).o_base, V, counts_in, alpha_bar, o_part, sm_o);
    else obar_chunk<T, D, false>(tab.unit(ui), c - tab.unit(ui).o_base, V, counts_in, alpha_bar, o_part, sm_o);
  }
}

__global__ void obar_reduce_kernel(const UnitTable tab, const Shape sh, const float* __restrict__ parts,
                                   float* __restrict__ o_bar) {
  obar_reduce_unit(tab.unit(blockIdx.x), sh, parts, o_bar);
}

__global__ void select_clear_kernel(unsigned int* sel_shared) {
  uint4* z = reinterpret_cast<uint4*>(sel_shared + (size_t)blockIdx.x * kSelSharedInts);
  for (int i = threadIdx.x; i < kSelSharedInts / 4; i += blockDim.x) z[i] = make_uint4(0u, 0u, 0u, 0u);
}

template <typename T, int D>
hipError_t launch_t(const UnitTable& tab, const Shape& sh, bool with_select, const float* alpha_bar,
                    uint8_t* edge_mask, int32_t* slot, const void* V, const int32_t* counts_in, float* o_part,
                    hipStream_t stream, const float* parts_in, float* o_bar_out, unsigned int* sel_shared) {
  const int n_select = with_select ? tab.total_sparts : 0;
  const int n_reduce = o_bar_out ? tab.n_units : 0;
  const int n_obar = V ? tab.total_ochunks : 0;
  if (n_select + n_reduce + n_obar == 0) return hipSuccess;
  if (with_select && tab.total_sparts != tab.n_units && sel_shared == nullptr) return hipErrorInvalidValue;
  // a part waits at most 200 us for the others (the clock of wall_clock64() runs at 100 MHz); KVS_DEBUG_SELECT_SPLIT = 3
  // makes that zero, so that the parts give up at their first wait and part 0 does the unit alone (a test of that way out)
  const unsigned timeout_ticks = debug_switch(KVS_DEBUG_SELECT_SPLIT) == 3 ? 0u : 20000u;
  // the small-LDS kernel when no unit needs more keys in one workgroup's LDS than it holds (a unit split into parts
  // does not; if its parts give up, its first part selects it from alpha_bar, pass by pass)
  bool small = true;
  for (int i = 0; with_select && i < tab.n_units; ++i) {
    const Unit un = tab.unit(i);
    const int parts = (i + 1 < tab.n_units ? tab.unit(i + 1).s_base : tab.total_sparts) - un.s_base;
    const int E = (un.len - 2 - sh.n_recent) - sh.n_sink + 1;
    if (parts == 1 && un.len > un.n_out && E + 6 > kLdsKeysSmall) small = false;
  }
  const dim3 grid(n_select + n_reduce + n_obar), block(kSelThreads);
  if (small) {
    hipLaunchKernelGGL((select_obar_kernel<T, D, kLdsKeysSmall>), grid, block, 0, stream, tab, sh, n_select, n_reduce,
                       alpha_bar, edge_mask, slot, (const T*)V, counts_in, o_part, parts_in, o_bar_out, sel_shared,
                       timeout_ticks);
  } else {
    hipLaunchKernelGGL((select_obar_kernel<T, D, kLdsKeys>), grid, block, 0, stream, tab, sh, n_select, n_reduce,
                       alpha_bar, edge_mask, slot, (const T*)V, counts_in, o_part, parts_in, o_bar_out, sel_shared,
                       timeout_ticks);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_select_clear(const UnitTable& tab, unsigned int* sel_shared, hipStream_t stream) {
  hipLaunchKernelGGL(select_clear_kernel, dim3(tab.n_units < kInlineUnits ? tab.n_units : kInlineUnits), dim3(256), 0, stream,
                     sel_shared);
  return hipGetLastError();
}

hipError_t launch_select_obar(const UnitTable& tab, const Shape& sh, kvs_dtype dt, bool with_select,
                              const float* alpha_bar, uint8_t* edge_mask, int32_t* slot, const void* V,
                              const int32_t* counts_in, float* o_part, hipStream_t stream, const float* parts_in,
                              float* o_bar_out, unsigned int* sel_shared) {
#define KVS_SEL_ARGS tab, sh, with_select, alpha_bar, edge_mask, slot, V, counts_in, o_part, stream, parts_in, o_bar_out, sel_shared
  if (dt == KVS_F32) return sh.D == 64 ? launch_t<float, 64>(KVS_SEL_ARGS) : launch_t<float, 128>(KVS_SEL_ARGS);
  return sh.D == 64 ? launch_t<uint16_t, 64>(KVS_SEL_ARGS) : launch_t<uint16_t, 128>(KVS_SEL_ARGS);
#undef KVS_SEL_ARGS
}

hipError_t launch_obar_reduce(const UnitTable& tab, const Shape& sh, const float* parts, float* o_bar,
                              hipStream_t stream) {
  hipLaunchKernelGGL(obar_reduce_kernel, dim3(tab.n_units), dim3(128), 0, stream, tab, sh, parts, o_bar);
  return hipGetLastError();
}

}  // namespace kvs
