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
// select (11 + 11 + 10 bits, LDS histograms) finds the r-th smallest key T and how many keys equal
// to T are still wanted; a final pass in index order takes every key below T and the first `want`
// keys equal to T, and turns the selection into the slot map with wavefront ballots and a scan
// over the 16 wavefronts.  Keys of units up to kLdsKeys edges are kept in LDS between the passes;
// longer units recompute them from alpha_bar (L2-resident).
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
constexpr int kLdsKeys = 32768;
constexpr int kBins = 2048;

__device__ __forceinline__ uint32_t edge_key(const float* __restrict__ a, int m) {
  return __float_as_uint(a[m] + a[m + 1]);
}

__device__ __forceinline__ int lanes_below(uint64_t ballot, int lane) {
  return __popcll(ballot & ((1ull << lane) - 1ull));
}

#ifdef KVS_TRACE_SEL
__device__ long long g_trace_sel[64 * 16];
#define KVS_SSTAMP(slot) do { if (threadIdx.x == 0) g_trace_sel[blockIdx.x * 16 + (slot)] = clock64(); } while (0)
#else
#define KVS_SSTAMP(slot) do { } while (0)
#endif

constexpr int kCand = 2048;               // keys of the first-pass bin that are refined in LDS

struct SelectSmem {
  uint32_t keys[kLdsKeys];
  uint32_t cand[kCand];
  int hist[kBins];
  int wave[kSelWaves];
  int pick[2];           // digit, keys below it
  int lt[kSelWaves], eq[kSelWaves];
  int ncand;
};

// Adds one to hist[d] for every active lane.  (Peeling groups of equal digits off with ballots before
// the atomics was measured and is slower than letting the LDS serialise equal addresses.)
__device__ __forceinline__ void hist_add(int* hist, uint32_t d, bool act, int lane) {
  (void)lane;
  if (act) atomicAdd(&hist[d], 1);
}

// Exclusive scan of the histogram (two bins per thread); finds the bin that holds rank `want`
// (1-based) and extends (prefix, pmask, want) by that digit.
__device__ __forceinline__ void pick_bin(SelectSmem& sm, int shift, int bins, uint32_t& prefix, uint32_t& pmask,
                                         int& want) {
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int h0 = sm.hist[2 * tid], h1 = sm.hist[2 * tid + 1];
  int incl = h0 + h1;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int v = __shfl_up(incl, off, kWave);
    if (lane >= off) incl += v;
  }
  if (lane == kWave - 1) sm.wave[wave] = incl;
  __syncthreads();
  int base = 0;
  for (int w = 0; w < wave; ++w) base += sm.wave[w];
  const int excl = base + incl - (h0 + h1);
  if (want > excl && want <= excl + h0) { sm.pick[0] = 2 * tid; sm.pick[1] = excl; }
  else if (want > excl + h0 && want <= excl + h0 + h1) { sm.pick[0] = 2 * tid + 1; sm.pick[1] = excl + h0; }
  __syncthreads();
  prefix |= (uint32_t)sm.pick[0] << shift;
  pmask |= (uint32_t)(bins - 1) << shift;
  want -= sm.pick[1];
  __syncthreads();
}

__device__ __forceinline__ void select_unit(const Unit& un, const Shape& sh, const float* __restrict__ alpha_bar,
                            uint8_t* __restrict__ edge_mask, int32_t* __restrict__ slot, SelectSmem& sm) {
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
  const bool cached = (E <= kLdsKeys);
  KVS_SSTAMP(0);

  // ---- keys (to LDS when they fit) and the histogram of their top 11 bits, four keys per thread at a
  //      time with the loads batched
  for (int b = tid; b < kBins; b += kSelThreads) sm.hist[b] = 0;
  if (tid == 0) sm.ncand = 0;
  __syncthreads();
  for (int base = 0; base < E; base += 4 * kSelThreads) {
    float x[4], y[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int m = lo + min(base + u * kSelThreads + tid, E - 1);
      x[u] = a[m];
      y[u] = a[m + 1];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = base + u * kSelThreads + tid;
      const uint32_t k = __float_as_uint(x[u] + y[u]);
      if (cached && i < E) sm.keys[i] = k;
      hist_add(sm.hist, k >> 21, i < E, lane);
    }
  }
  if (cached && tid < 4 && E + tid < ((E + 3) & ~3)) sm.keys[E + tid] = 0xffffffffu;   // pad to groups of four
  __syncthreads();
  uint32_t prefix = 0, pmask = 0;
  int want = r;                        // rank (1-based) among the keys that share `prefix`
  KVS_SSTAMP(1);
  pick_bin(sm, 21, 2048, prefix, pmask, want);
  KVS_SSTAMP(2);

  // ---- the keys of that bin go to a short list; the remaining 21 bits are settled on the list
  // (cached keys are scanned four at a time with 16-byte LDS reads: a quarter of the loop overhead)
  const uint4* k4 = reinterpret_cast<const uint4*>(sm.keys);
  const int G = (E + 3) / 4;           // groups of four keys
  if (cached) {
    for (int g = tid; g < G; g += kSelThreads) {
      const uint4 q = k4[g];
      const uint32_t kk[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if ((kk[u] & pmask) == prefix && 4 * g + u < E) {
          const int pos = atomicAdd(&sm.ncand, 1);
          if (pos < kCand) sm.cand[pos] = kk[u];
        }
      }
    }
  } else {
    for (int i = tid; i < E; i += kSelThreads) {
      const uint32_t k = edge_key(a, lo + i);
      if ((k & pmask) == prefix) {
        const int pos = atomicAdd(&sm.ncand, 1);
        if (pos < kCand) sm.cand[pos] = k;
      }
    }
  }
  __syncthreads();
  const int ncand = sm.ncand;
  KVS_SSTAMP(3);
  const bool listed = (ncand <= kCand);
  const int shifts[2] = {10, 0};
  const int widths[2] = {11, 10};
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
      for (int i = tid; i < E; i += kSelThreads) {
        const uint32_t k = cached ? sm.keys[i] : edge_key(a, lo + i);
        hist_add(sm.hist, (k >> shift) & (bins - 1), (k & pmask) == prefix, lane);
      }
    }
    __syncthreads();
    pick_bin(sm, shift, bins, prefix, pmask, want);
  }
  const uint32_t T = prefix;           // `want` keys equal to T are taken, the lowest indices first
  KVS_SSTAMP(4);

  // ---- ordered pass: every wavefront owns a contiguous range of edges
  if (cached) {
    // four consecutive keys per lane: wavefront w owns groups [g0, g1)
    const int per_g = ((G + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
    const int g0 = min(G, wave * per_g), g1 = min(G, g0 + per_g);
    int n_lt = 0, n_eq = 0;
    for (int g = g0 + lane; g < g1; g += kWave) {
      const uint4 q = k4[g];
      n_lt += (q.x < T) + (q.y < T) + (q.z < T) + (q.w < T);
      n_eq += (q.x == T && 4 * g < E) + (q.y == T && 4 * g + 1 < E) + (q.z == T && 4 * g + 2 < E) +
              (q.w == T && 4 * g + 3 < E);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      n_lt += __shfl_xor(n_lt, off, kWave);
      n_eq += __shfl_xor(n_eq, off, kWave);
    }
    if (lane == 0) { sm.lt[wave] = n_lt; sm.eq[wave] = n_eq; }
    __syncthreads();
    KVS_SSTAMP(5);
    int eq_before = 0, sel_before = 0;
    for (int w = 0; w < wave; ++w) {
      const int take = min(max(want - eq_before, 0), sm.eq[w]);
      sel_before += sm.lt[w] + take;
      eq_before += sm.eq[w];
    }
    const bool vec_ok = ((un.in_row + lo) & 3) == 0;       // 4-byte mask stores and 16-byte slot stores
    for (int gb = g0; gb < g1; gb += kWave) {              // whole wavefront iterates together
      const int g = gb + lane;
      uint4 q = make_uint4(0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu);
      if (g < g1) q = k4[g];
      const uint32_t kk[4] = {q.x, q.y, q.z, q.w};
      bool sel[4], eq[4];
      int lane_eq = 0;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        sel[u] = kk[u] < T;
        eq[u] = (kk[u] == T) && (4 * g + u < E) && (g < g1);
        lane_eq += eq[u];
      }
      if (__ballot(lane_eq != 0) != 0) {                  // ties with the threshold: rare, ranked in index order
        int incl = lane_eq;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
          const int v = __shfl_up(incl, off, kWave);
          if (lane >= off) incl += v;
        }
        int rank = eq_before + incl - lane_eq;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (eq[u]) { sel[u] = rank < want; ++rank; }
        }
        eq_before += __shfl(incl, kWave - 1, kWave);
      }
      const int lane_cnt = sel[0] + sel[1] + sel[2] + sel[3];
      int incl = lane_cnt;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const int v = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += v;
      }
      int below = sel_before + incl - lane_cnt;              // selected edges below this lane's first key
      sel_before += __shfl(incl, kWave - 1, kWave);
      if (g < g1) {
        const int m0 = lo + 4 * g;
        int s4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) { s4[u] = m0 + u - below; below += sel[u]; }
        if (vec_ok && 4 * g + 3 < E) {
          *reinterpret_cast<uint32_t*>(mk + m0) =
              (uint32_t)sel[0] | ((uint32_t)sel[1] << 8) | ((uint32_t)sel[2] << 16) | ((uint32_t)sel[3] << 24);
          *reinterpret_cast<int4*>(sl + m0) = make_int4(s4[0], s4[1], s4[2], s4[3]);
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            if (4 * g + u < E) { mk[m0 + u] = sel[u] ? 1 : 0; sl[m0 + u] = s4[u]; }
          }
        }
      }
    }
  } else {
    const int per = ((E + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
    const int e0 = min(E, wave * per), e1 = min(E, e0 + per);
    int n_lt = 0, n_eq = 0;
    for (int i = e0 + lane; i < e1 + lane; i += kWave) {     // whole wavefront iterates together
      uint32_t k = 0xffffffffu;
      if (i < e1) k = edge_key(a, lo + i);
      n_lt += __popcll(__ballot(k < T));
      n_eq += __popcll(__ballot(k == T && i < e1));
    }
    if (lane == 0) { sm.lt[wave] = n_lt; sm.eq[wave] = n_eq; }
    __syncthreads();
    int eq_before = 0, sel_before = 0;
    for (int w = 0; w < wave; ++w) {
      const int take = min(max(want - eq_before, 0), sm.eq[w]);
      sel_before += sm.lt[w] + take;
      eq_before += sm.eq[w];
    }
    for (int i = e0 + lane; i < e1 + lane; i += kWave) {
      uint32_t k = 0xffffffffu;
      if (i < e1) k = edge_key(a, lo + i);
      const bool is_eq = (k == T) && (i < e1);
      const uint64_t beq = __ballot(is_eq);
      const bool sel = (k < T) || (is_eq && (eq_before + lanes_below(beq, lane) < want));
      const uint64_t bsel = __ballot(sel);
      if (i < e1) {
        const int m = lo + i;
        mk[m] = sel ? 1 : 0;
        sl[m] = m - (sel_before + lanes_below(bsel, lane));   // selected edges below token m
      }
      eq_before += __popcll(beq);
      sel_before += __popcll(bsel);
    }
  }
  // tokens outside the eligible edge range
  for (int t = tid; t < lo && t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t; }
  for (int t = hi + 1 + tid; t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t - r; }
  KVS_SSTAMP(6);
}

template <typename T, int D>
__device__ __forceinline__ void obar_chunk(const Unit& un, int chunk, const T* __restrict__ V, const float* __restrict__ alpha_bar,
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
      raw[u] = Vp[(size_t)tc * LPR];
      a[u] = (t < t1) ? al[tc] : 0.f;
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

template <typename T, int D>
__global__ __launch_bounds__(kSelThreads) void select_obar_kernel(
    const UnitTable tab, const Shape sh, const int n_select, const float* __restrict__ alpha_bar,
    uint8_t* __restrict__ edge_mask, int32_t* __restrict__ slot, const T* __restrict__ V,
    float* __restrict__ o_part) {
  __shared__ SelectSmem sm;
  __shared__ float sm_o[kSelWaves][128];
  const int b = blockIdx.x;
  if (b < n_select) {
    select_unit(tab.u[b], sh, alpha_bar, edge_mask, slot, sm);
  } else {
    const int c = b - n_select;
    int ui = 0;
    while (ui + 1 < tab.n_units && tab.u[ui + 1].o_base <= c) ++ui;
    obar_chunk<T, D>(tab.u[ui], c - tab.u[ui].o_base, V, alpha_bar, o_part, sm_o);
  }
}

__global__ void obar_reduce_kernel(const UnitTable tab, const Shape sh, const float* __restrict__ o_part,
                                   float* __restrict__ o_bar) {
  const Unit un = tab.u[blockIdx.x];
  const int nc = obar_chunks(un.len);
  for (int d = threadIdx.x; d < sh.D; d += blockDim.x) {
    float s = 0.f;
    for (int c = 0; c < nc; ++c) s += o_part[((size_t)un.index * kMaxChunks + c) * sh.D + d];
    o_bar[(size_t)un.index * sh.D + d] = s;
  }
}

template <typename T, int D>
hipError_t launch_t(const UnitTable& tab, const Shape& sh, bool with_select, const float* alpha_bar,
                    uint8_t* edge_mask, int32_t* slot, const void* V, float* o_part, hipStream_t stream) {
  const int n_select = with_select ? tab.n_units : 0;
  const int n_obar = V ? tab.total_ochunks : 0;
  if (n_select + n_obar == 0) return hipSuccess;
  hipLaunchKernelGGL((select_obar_kernel<T, D>), dim3(n_select + n_obar), dim3(kSelThreads), 0, stream, tab, sh,
                     n_select, alpha_bar, edge_mask, slot, (const T*)V, o_part);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_select_obar(const UnitTable& tab, const Shape& sh, kvs_dtype dt, bool with_select,
                              const float* alpha_bar, uint8_t* edge_mask, int32_t* slot, const void* V,
                              float* o_part, hipStream_t stream) {
  if (dt == KVS_F32) {
    return sh.D == 64 ? launch_t<float, 64>(tab, sh, with_select, alpha_bar, edge_mask, slot, V, o_part, stream)
                      : launch_t<float, 128>(tab, sh, with_select, alpha_bar, edge_mask, slot, V, o_part, stream);
  }
  return sh.D == 64 ? launch_t<uint16_t, 64>(tab, sh, with_select, alpha_bar, edge_mask, slot, V, o_part, stream)
                    : launch_t<uint16_t, 128>(tab, sh, with_select, alpha_bar, edge_mask, slot, V, o_part, stream);
}

hipError_t launch_obar_reduce(const UnitTable& tab, const Shape& sh, const float* o_part, float* o_bar,
                              hipStream_t stream) {
  hipLaunchKernelGGL(obar_reduce_kernel, dim3(tab.n_units), dim3(128), 0, stream, tab, sh, o_part, o_bar);
  return hipGetLastError();
}

#ifdef KVS_TRACE_SEL
extern "C" int kvs_debug_trace_sel(void* host, size_t bytes) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace_sel), bytes);
}
#endif

}  // namespace kvs
