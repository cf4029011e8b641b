// Select kernel: which adjacent pairs merge, and the slot of every token.
//
// Per unit: edge score sigma[m] = alpha_bar[m] + alpha_bar[m+1] for the eligible edges
// n_sink <= m <= len-2-n_recent (App. C, paragraph (i): pairs with small accumulated attention
// mass; Sec. 5: the first tokens are always preserved); the r = len - budget smallest scores are
// selected in one parallel step (Sec. 3.1), ties going to the lower index; consecutive selected
// edges chain into one output slot.
//
// One workgroup of 1024 threads per unit.  Scores are non-negative floats, so their bit patterns
// order like unsigned integers: an MSB-first radix select (11 + 11 + 10 bits, LDS histograms)
// finds the r-th smallest key T and how many keys equal to T are still wanted; a final pass in
// index order takes every key below T and the first `want` keys equal to T, and turns the
// selection into the slot map with wavefront ballots and a scan over the 16 wavefronts.  Keys of
// units up to kLdsKeys edges are kept in LDS between the passes; longer units recompute them from
// alpha_bar (L2-resident).
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

__global__ __launch_bounds__(kSelThreads) void select_kernel(
    const UnitTable tab, const Shape sh, const float* __restrict__ alpha_bar, uint8_t* __restrict__ edge_mask,
    int32_t* __restrict__ slot, const float* __restrict__ o_part, float* __restrict__ o_bar) {
  __shared__ uint32_t sm_keys[kLdsKeys];
  __shared__ int sm_hist[kBins];
  __shared__ int sm_wave[kSelWaves];
  __shared__ int sm_pick[2];           // digit, keys below it
  __shared__ int sm_lt[kSelWaves], sm_eq[kSelWaves];

  const Unit un = tab.u[blockIdx.x];
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int n = un.len;
  const int r = n - un.n_out;
  const float* a = alpha_bar + un.in_row;
  uint8_t* mk = edge_mask + un.in_row;
  int32_t* sl = slot + un.in_row;

  if (o_part != nullptr) {             // fused: o_bar = sum of the chunks' partial sums, in chunk order
    for (int d = tid; d < sh.D; d += kSelThreads) {
      float s = 0.f;
      for (int c = 0; c < un.n_chunks; ++c) s += o_part[((size_t)un.index * kMaxChunks + c) * sh.D + d];
      o_bar[(size_t)un.index * sh.D + d] = s;
    }
  }

  const int lo = sh.n_sink;
  const int hi = n - 2 - sh.n_recent;
  const int E = hi - lo + 1;           // eligible edges; the host has checked r <= E whenever r > 0
  if (r <= 0 || E <= 0) {
    for (int t = tid; t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t; }
    return;
  }
  const bool cached = (E <= kLdsKeys);
  if (cached) {
    for (int i = tid; i < E; i += kSelThreads) sm_keys[i] = edge_key(a, lo + i);
  }
  __syncthreads();

  // ---- radix select of the r-th smallest key
  uint32_t prefix = 0, pmask = 0;
  int want = r;                        // rank (1-based) among the keys that share `prefix`
  const int shifts[3] = {21, 10, 0};
  const int widths[3] = {11, 11, 10};
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = shifts[pass];
    const int bins = 1 << widths[pass];
    for (int b = tid; b < kBins; b += kSelThreads) sm_hist[b] = 0;
    __syncthreads();
    for (int i = tid; i < E; i += kSelThreads) {
      const uint32_t k = cached ? sm_keys[i] : edge_key(a, lo + i);
      if ((k & pmask) == prefix) atomicAdd(&sm_hist[(k >> shift) & (bins - 1)], 1);
    }
    __syncthreads();
    // exclusive scan over the bins, two bins per thread
    const int h0 = sm_hist[2 * tid], h1 = sm_hist[2 * tid + 1];
    int incl = h0 + h1;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int v = __shfl_up(incl, off, kWave);
      if (lane >= off) incl += v;
    }
    if (lane == kWave - 1) sm_wave[wave] = incl;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += sm_wave[w];
    const int excl = base + incl - (h0 + h1);
    if (want > excl && want <= excl + h0) { sm_pick[0] = 2 * tid; sm_pick[1] = excl; }
    else if (want > excl + h0 && want <= excl + h0 + h1) { sm_pick[0] = 2 * tid + 1; sm_pick[1] = excl + h0; }
    __syncthreads();
    prefix |= (uint32_t)sm_pick[0] << shift;
    pmask |= (uint32_t)(bins - 1) << shift;
    want -= sm_pick[1];
    __syncthreads();
  }
  const uint32_t T = prefix;           // `want` keys equal to T are taken, the lowest indices first

  // ---- ordered pass: every wavefront owns a contiguous range of edges
  const int per = ((E + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
  const int e0 = min(E, wave * per), e1 = min(E, e0 + per);
  int n_lt = 0, n_eq = 0;
  for (int i = e0 + lane; i < e1 + lane; i += kWave) {     // whole wavefront iterates together
    uint32_t k = 0xffffffffu;
    if (i < e1) k = cached ? sm_keys[i] : edge_key(a, lo + i);
    n_lt += __popcll(__ballot(k < T));
    n_eq += __popcll(__ballot(k == T && i < e1));
  }
  if (lane == 0) { sm_lt[wave] = n_lt; sm_eq[wave] = n_eq; }
  __syncthreads();
  int eq_before = 0, sel_before = 0;
  for (int w = 0; w < wave; ++w) {
    const int take = min(max(want - eq_before, 0), sm_eq[w]);
    sel_before += sm_lt[w] + take;
    eq_before += sm_eq[w];
  }
  for (int i = e0 + lane; i < e1 + lane; i += kWave) {
    uint32_t k = 0xffffffffu;
    if (i < e1) k = cached ? sm_keys[i] : edge_key(a, lo + i);
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
  // tokens outside the eligible edge range
  for (int t = tid; t < lo && t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t; }
  for (int t = hi + 1 + tid; t < n; t += kSelThreads) { mk[t] = 0; sl[t] = t - r; }
}

}  // namespace

hipError_t launch_select(const UnitTable& tab, const Shape& sh, const float* alpha_bar, uint8_t* edge_mask,
                         int32_t* slot, const Workspace* ws_for_obar, float* o_bar, hipStream_t stream) {
  hipLaunchKernelGGL(select_kernel, dim3(tab.n_units), dim3(kSelThreads), 0, stream, tab, sh, alpha_bar,
                     edge_mask, slot, ws_for_obar ? ws_for_obar->o_part : nullptr, o_bar);
  return hipGetLastError();
}

}  // namespace kvs
