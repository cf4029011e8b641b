// Per-query aggregation of the sensitivity norms, fp32 inputs (vector ALU).
//
// The same quantities as the bf16 kernels of kvs_perquery.hip: every query row q keeps its own attention
// alpha^{(q)} and its own output o^{(q)} (Sec. 4.1, Eq. attn_def_vec), the vectors of Eqs. c11_def-c12_def are
// formed per row, and their norms are averaged over the R rows:
//   A_t = (1/R) sum_q alpha_t^{(q)} |1 - 2 alpha_t^{(q)}| ||v_t - o^{(q)}||
//   C_t = (1/R) sum_q alpha_t^{(q)} alpha_{t+1}^{(q)} ||v_t + v_{t+1} - 2 o^{(q)}||
// fp32 caches are the small configurations, so these kernels are written for any shape rather than for speed:
// all arithmetic is fp32 on the vector ALU, the squared distances are taken directly (sum of squared
// differences, no expansion), units may be shorter than a tile, and there is no limit on R.
// counts_in (or null): the rows are slots of an already merged cache (Sec. 3.1, streaming regime), row t standing
// for c_t tokens whose Values add up to V[t]; every query row then sees it as one token with logit e + ln c_t and
// value V[t] / c_t.
//
// Three kernels after the two score sweeps (which leave the normaliser c[q] of every row):
//   pq_out_f32_kernel     o_part[chunk, q, :] = sum over the chunk's tokens of (alpha_t^{(q)} / R) V[t], and
//                         p_part[chunk, q] = the sum of the same weights alpha_t^{(q)} / R
//   pq_reduce_f32_kernel  o^{(q)} = (sum of the o_part) / (sum of the p_part), in chunk order: a convex combination
//                         of the Values with the weights as they were rounded, so that where a row puts nearly all
//                         its weight on one token, o - v_t is as accurate as the small weights of the others
//                         (dividing by the weights' nominal sum 1 / R leaves the rounding of the normaliser c[q],
//                         which grows with the logits, times ||v_t||)
//   pq_norms_f32_kernel   A_t and C_t of the chunk's tokens
// A workgroup walks its chunk in tiles of 32 tokens held in LDS and takes the query rows eight at a time:
// thread (q, t) = (tid / 32, tid % 32) owns one (query row, token) pair.  Sums run in fixed orders; no atomics.
#include "kvs_device.h"

namespace kvs {
namespace {

constexpr int kThreads = 256;
constexpr int kTile = 32;             // tokens per tile
constexpr int kQB = kThreads / kTile; // query rows per block: 8

template <int D>
struct Lds {
  static constexpr int STRIDE = D + 4;          // floats per row: 16-byte pieces of neighbouring rows fall in different banks
};

// rows [row0, row0 + nrows) of a row-major [.., D] matrix -> LDS (rows at or beyond `limit` become zeros)
template <int D>
__device__ __forceinline__ void load_rows(float* sm, const float* __restrict__ g, long long row0, int nrows,
                                          long long limit, int tid) {
  constexpr int PPR = D / 4;
  for (int i = tid; i < nrows * PPR; i += kThreads) {
    const int r = i / PPR, p = i % PPR;
    float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row0 + r < limit) x = *reinterpret_cast<const float4*>(g + (size_t)(row0 + r) * D + 4 * p);
    *reinterpret_cast<float4*>(sm + r * Lds<D>::STRIDE + 4 * p) = x;
  }
}

// log2 c and 1 / c of the rows [row0, row0 + nrows) -> LDS (1 for plain tokens and for rows at or beyond `limit`)
__device__ __forceinline__ void load_counts(float* sm_lc, float* sm_ic, const int32_t* __restrict__ cnt, long long row0,
                                            int nrows, long long limit, int tid) {
  if (tid < nrows) {
    const float c = (cnt != nullptr && row0 + tid < limit) ? (float)cnt[row0 + tid] : 1.f;
    sm_lc[tid] = __builtin_amdgcn_logf(c);         // (the hardware's base-2 logarithm)
    sm_ic[tid] = __builtin_amdgcn_rcpf(c);
  }
}

template <int D>
__device__ __forceinline__ float dot_rows(const float* a, const float* b) {
  float s = 0.f;
#pragma unroll
  for (int d = 0; d < D; d += 4) {
    const float4 x = *reinterpret_cast<const float4*>(a + d);
    const float4 y = *reinterpret_cast<const float4*>(b + d);
    s = fmaf(x.x, y.x, s); s = fmaf(x.y, y.y, s); s = fmaf(x.z, y.z, s); s = fmaf(x.w, y.w, s);
  }
  return s;
}

// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads) void pq_out_f32_kernel(const UnitTable tab, const Shape sh,
                                                              const float* __restrict__ Q, const float* __restrict__ K,
                                                              const float* __restrict__ V,
                                                              const int32_t* __restrict__ counts_in,
                                                              const float* __restrict__ c_row,
                                                              float* __restrict__ o_part, float* __restrict__ p_part) {
  constexpr int S = Lds<D>::STRIDE;
  constexpr int DPT = D / kTile;                 // output dimensions per thread
  __shared__ float sm_lc[kTile + 1], sm_ic[kTile + 1];
  __shared__ __attribute__((aligned(16))) float sm_k[kTile * S];
  __shared__ __attribute__((aligned(16))) float sm_v[kTile * S];
  __shared__ __attribute__((aligned(16))) float sm_q[kQB * S];
  __shared__ float2 sm_p[kQB][kTile];            // (alpha / R, the same divided by the row's cardinality)

  const int ui = find_unit(tab, blockIdx.x);
  const Unit un = tab.unit(ui);
  const int chunk = blockIdx.x - un.chunk_base;
  const int t0 = chunk * un.chunk_len;
  const int t1 = min(un.len, t0 + un.chunk_len);
  const int tid = threadIdx.x, ql = tid / kTile, tl = tid % kTile;
  const int R = sh.R;
  const float* Kg = K + (size_t)un.in_row * D;
  const float* Vg = V + (size_t)un.in_row * D;
  const float* Qu = Q + (size_t)un.index * R * D;
  const int32_t* cnt = counts_in ? counts_in + un.in_row : nullptr;

  for (int qb = 0; qb < R; qb += kQB) {
    const int q = qb + ql;
    __syncthreads();                              // the block before has finished with sm_q
    load_rows<D>(sm_q, Qu, qb, kQB, R, tid);
    const float cq = (q < R) ? c_row[(size_t)un.index * R + q] : INFINITY;      // exp2(-inf) = 0: no such row
    const int lim = last_seen_row(sh.causal, un.len, q);
    float acc[DPT];
#pragma unroll
    for (int i = 0; i < DPT; ++i) acc[i] = 0.f;
    float wsum = 0.f;                             // (every thread of the row adds the same weights in the same order)
    for (int tb = t0; tb < t1; tb += kTile) {
      __syncthreads();                            // the tile before has been used up
      load_rows<D>(sm_k, Kg, tb, kTile, t1, tid);
      load_rows<D>(sm_v, Vg, tb, kTile, t1, tid);
      load_counts(sm_lc, sm_ic, cnt, tb, kTile, t1, tid);
      __syncthreads();
      const int t = tb + tl;
      const float x = dot_rows<D>(sm_q + ql * S, sm_k + tl * S);
      // alpha / R, and (alpha / R) / c: the row's weight for the Value SUM V[t]
      const float w = (t < t1 && t <= lim) ? __builtin_amdgcn_exp2f(fmaf(x, sh.scale_log2, sm_lc[tl] - cq)) : 0.f;
      sm_p[ql][tl] = make_float2(w, w * sm_ic[tl]);
      __syncthreads();
#pragma unroll 4
      for (int r = 0; r < kTile; ++r) {
        const float2 p = sm_p[ql][r];
        wsum += p.x;
#pragma unroll
        for (int i = 0; i < DPT; ++i) acc[i] = fmaf(p.y, sm_v[r * S + tl + kTile * i], acc[i]);
      }
    }
    if (q < R) {
      float* dst = o_part + ((size_t)(un.chunk_base + chunk) * R + q) * D;
#pragma unroll
      for (int i = 0; i < DPT; ++i) dst[tl + kTile * i] = acc[i];
      if (tl == 0) p_part[(size_t)(un.chunk_base + chunk) * R + q] = wsum;
    }
  }
}

// o[unit, q, :] = (sum of the chunk partials) / (sum of their weights), both in chunk order.  One workgroup of D
// threads per (unit, row).
template <int D>
__global__ __launch_bounds__(D) void pq_reduce_f32_kernel(const UnitTable tab, const Shape sh,
                                                          const float* __restrict__ o_part,
                                                          const float* __restrict__ p_part, float* __restrict__ o) {
  const int R = sh.R;
  const Unit un = tab.unit(blockIdx.x / R);
  const int q = blockIdx.x % R;
  const int d = threadIdx.x;
  float s = 0.f, w = 0.f;
  for (int c = 0; c < un.n_chunks; ++c) {
    s += o_part[((size_t)(un.chunk_base + c) * R + q) * D + d];
    w += p_part[(size_t)(un.chunk_base + c) * R + q];
  }
  o[((size_t)un.index * R + q) * D + d] = s / w;
}

// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads) void pq_norms_f32_kernel(const UnitTable tab, const Shape sh,
                                                                const float* __restrict__ Q,
                                                                const float* __restrict__ K,
                                                                const float* __restrict__ V,
                                                                const int32_t* __restrict__ counts_in,
                                                                const float* __restrict__ c_row,
                                                                const float* __restrict__ o, float* __restrict__ a_tok,
                                                                float* __restrict__ c_edge) {
  constexpr int S = Lds<D>::STRIDE;
  __shared__ __attribute__((aligned(16))) float sm_k[(kTile + 1) * S];   // one row more: the last token's neighbour
  __shared__ __attribute__((aligned(16))) float sm_v[(kTile + 1) * S];
  __shared__ __attribute__((aligned(16))) float sm_q[kQB * S];
  __shared__ __attribute__((aligned(16))) float sm_o[kQB * S];
  __shared__ float sm_a[kQB][kTile + 1];          // alpha / R of the block's rows at the tile's tokens
  __shared__ float2 sm_r[kQB][kTile];             // the rows' shares of A_t and C_t
  __shared__ float sm_lc[kTile + 1], sm_ic[kTile + 1];

  const int ui = find_unit(tab, blockIdx.x);
  const Unit un = tab.unit(ui);
  const int chunk = blockIdx.x - un.chunk_base;
  const int t0 = chunk * un.chunk_len;
  const int t1 = min(un.len, t0 + un.chunk_len);
  const int tid = threadIdx.x, ql = tid / kTile, tl = tid % kTile;
  const int R = sh.R;
  const float Rf = (float)R;
  const float* Kg = K + (size_t)un.in_row * D;
  const float* Vg = V + (size_t)un.in_row * D;
  const float* Qu = Q + (size_t)un.index * R * D;
  const float* Ou = o + (size_t)un.index * R * D;
  const int32_t* cnt = counts_in ? counts_in + un.in_row : nullptr;

  for (int tb = t0; tb < t1; tb += kTile) {
    __syncthreads();
    load_rows<D>(sm_k, Kg, tb, kTile + 1, un.len, tid);      // the neighbour of the chunk's last token is the next chunk's first
    load_rows<D>(sm_v, Vg, tb, kTile + 1, un.len, tid);
    load_counts(sm_lc, sm_ic, cnt, tb, kTile + 1, un.len, tid);
    const int t = tb + tl;
    float sumA = 0.f, sumC = 0.f;                  // threads 0..31: token tl of the tile, over all query rows
    for (int qb = 0; qb < R; qb += kQB) {
      const int q = qb + ql;
      __syncthreads();                             // the tile is in place; the block before is done with sm_q, sm_o, sm_r
      load_rows<D>(sm_q, Qu, qb, kQB, R, tid);
      load_rows<D>(sm_o, Ou, qb, kQB, R, tid);
      __syncthreads();
      const float cq = (q < R) ? c_row[(size_t)un.index * R + q] : INFINITY;
      const int lim = last_seen_row(sh.causal, un.len, q);
      const float* qrow = sm_q + ql * S;
      const float x = dot_rows<D>(qrow, sm_k + tl * S);
      const float a = (t < un.len && t <= lim) ? __builtin_amdgcn_exp2f(fmaf(x, sh.scale_log2, sm_lc[tl] - cq)) : 0.f;
      sm_a[ql][tl] = a;
      if (tl == kTile - 1) {                       // the tile's extra row
        const float xn = dot_rows<D>(qrow, sm_k + kTile * S);
        sm_a[ql][kTile] = (t + 1 < un.len && t + 1 <= lim)
                              ? __builtin_amdgcn_exp2f(fmaf(xn, sh.scale_log2, sm_lc[kTile] - cq)) : 0.f;
      }
      float d2 = 0.f, p2 = 0.f;                    // ||v_t - o||^2, ||v_t + v_{t+1} - 2o||^2 with v = V / c
      const float* vt = sm_v + tl * S;
      const float* orow = sm_o + ql * S;
      const float ic0 = sm_ic[tl], ic1 = sm_ic[tl + 1];
#pragma unroll 2
      for (int d = 0; d < D; d += 4) {
        const float4 v0 = *reinterpret_cast<const float4*>(vt + d);
        const float4 v1 = *reinterpret_cast<const float4*>(vt + S + d);
        const float4 oq = *reinterpret_cast<const float4*>(orow + d);
        const float r0[4] = {fmaf(v0.x, ic0, -oq.x), fmaf(v0.y, ic0, -oq.y), fmaf(v0.z, ic0, -oq.z), fmaf(v0.w, ic0, -oq.w)};
        const float r1[4] = {fmaf(v1.x, ic1, -oq.x), fmaf(v1.y, ic1, -oq.y), fmaf(v1.z, ic1, -oq.z), fmaf(v1.w, ic1, -oq.w)};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          d2 = fmaf(r0[i], r0[i], d2);
          const float s = r0[i] + r1[i];
          p2 = fmaf(s, s, p2);
        }
      }
      __syncthreads();
      const float a_n = sm_a[ql][tl + 1];
      sm_r[ql][tl] = make_float2(a * fabsf(fmaf(-2.f * Rf, a, 1.f)) * __builtin_amdgcn_sqrtf(d2),
                                 a * a_n * __builtin_amdgcn_sqrtf(p2));
      __syncthreads();
      if (tid < kTile) {
#pragma unroll
        for (int r = 0; r < kQB; ++r) {            // rows beyond R have a = 0
          sumA += sm_r[r][tid].x;
          sumC += sm_r[r][tid].y;
        }
      }
    }
    if (tid < kTile && t < t1) {
      a_tok[un.in_row + t] = sumA;
      c_edge[un.in_row + t] = (t == un.len - 1) ? 0.f : sumC * Rf;
    }
  }
}

template <int D>
hipError_t launch_t(const UnitTable& tab, const Shape& sh, const float* Q, const float* K, const float* V,
                    const int32_t* counts_in, const float* c_row, float* o_part, float* o, float* a_tok, float* c_edge,
                    hipStream_t stream) {
  const dim3 grid(tab.total_chunks), block(kThreads);
  float* p_part = o_part + (size_t)tab.total_chunks * sh.R * D;   // the weights' sums lie behind the launch's partials
  hipLaunchKernelGGL((pq_out_f32_kernel<D>), grid, block, 0, stream, tab, sh, Q, K, V, counts_in, c_row, o_part,
                     p_part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((pq_reduce_f32_kernel<D>), dim3(tab.n_units * sh.R), dim3(D), 0, stream, tab, sh, o_part, p_part,
                     o);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((pq_norms_f32_kernel<D>), grid, block, 0, stream, tab, sh, Q, K, V, counts_in, c_row, o, a_tok,
                     c_edge);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_per_query_norms_f32(const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                                      const void* V, const int32_t* counts_in, const float* c_row, float* o_part,
                                      float* o, float* a_tok, float* c_edge, hipStream_t stream) {
  const float* q = (const float*)Q;
  const float* k = (const float*)K;
  const float* v = (const float*)V;
  return sh.D == 64 ? launch_t<64>(tab, sh, q, k, v, counts_in, c_row, o_part, o, a_tok, c_edge, stream)
                    : launch_t<128>(tab, sh, q, k, v, counts_in, c_row, o_part, o, a_tok, c_edge, stream);
}

}  // namespace kvs
