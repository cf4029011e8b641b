// Decode attention over a merged cache (the consumer of kvs_merge_compact's outputs).
//
// A row (k', V', c) of a merged cache stands for c tokens that all carry the Key k' and whose Values
// add up to V' (Sec. 3.1: the pair (k_m, k_{m+1}) is replaced by (k, k), the Values are summed, and the
// cardinality is carried along).  Attention of a query q over such a cache is
//   o = sum_S exp(e_S) V'_S / sum_S c_S exp(e_S),      e_S = scale * q . k'_S,
// i.e. ordinary attention over the c_S copies of every slot.  With c = 1 it is plain attention.
//
// Split over the rows of a unit (chunks of at least 512 rows, at most 64 per unit, one workgroup
// each; the grid is chunks x units): LPR adjacent lanes read one K row and one V row (16 bytes each), four query rows at a time
// sit in registers, every lane group keeps an online softmax (running maximum, denominator,
// D-wide numerator) for its rows, the groups of a workgroup are combined through LDS, and a second
// small kernel combines the chunks.  Everything is ordered: no atomics, results do not depend on
// timing.  The kernel is meant for decode-sized query blocks (at most KVS_MAX_DECODE_ROWS rows per
// unit); it reads the cache once per block of four query rows.
#include <algorithm>

#include "kvs_device.h"

namespace kvs {
namespace {

constexpr int kThreads = 256;
constexpr int kQB = 4;                    // query rows per block
constexpr int kUnroll = 2;                // cache rows per lane group in flight
#ifndef KVS_DEC_CHUNK
#define KVS_DEC_CHUNK 512
#endif
constexpr int kDecMinChunk = KVS_DEC_CHUNK;   // rows per workgroup, at least

// Chunking of a unit's rows: a function of its length only.
__host__ __device__ inline int dec_chunk_len(int len) {
  const int per = (len + kMaxChunks - 1) / kMaxChunks;
  const int rounded = (per + kWave - 1) / kWave * kWave;
  return rounded > kDecMinChunk ? rounded : kDecMinChunk;
}
__host__ __device__ inline int dec_chunks(int len) {
  const int cl = dec_chunk_len(len);
  return (len + cl - 1) / cl;
}

// partial result of one (unit, chunk, query row): numerator[D], running maximum, denominator
__device__ __forceinline__ size_t part_index(int unit_index, int chunk, int R, int row, int D) {
  return (((size_t)unit_index * kMaxChunks + chunk) * R + row) * (size_t)(D + 2);
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_partial_kernel(
    const UnitTable tab, const Shape sh, const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ counts, float* __restrict__ part) {
  constexpr int EPL = Piece<T>::N;
  constexpr int LPR = D / EPL;
  constexpr int RPW = kWave / LPR;
  constexpr int GROUPS = RPW * (kThreads / kWave);       // lane groups (= rows in flight) per workgroup

  __shared__ float sm_acc[GROUPS][kQB][D];
  __shared__ float2 sm_ml[GROUPS][kQB];

  const Unit un = tab.u[blockIdx.y];
  const int chunk = blockIdx.x;
  if (chunk >= dec_chunks(un.len)) return;               // the grid is as wide as the longest unit needs
  const int clen = dec_chunk_len(un.len);
  const int t0 = chunk * clen;
  const int t1 = min(un.len, t0 + clen);
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int grp = lane / LPR, piece = lane % LPR;
  const int group = wave * RPW + grp;
  const int R = sh.R;

  const uint4* Kp = reinterpret_cast<const uint4*>(K + (size_t)un.in_row * D) + piece;
  const uint4* Vp = reinterpret_cast<const uint4*>(V + (size_t)un.in_row * D) + piece;
  const uint4* Qp = reinterpret_cast<const uint4*>(Q + (size_t)un.index * R * D) + piece;
  const int32_t* cnt = counts ? counts + un.in_row : nullptr;

  for (int qb = 0; qb < R; qb += kQB) {
    float qf[kQB][EPL];
#pragma unroll
    for (int j = 0; j < kQB; ++j) {
      const uint4 raw = Qp[(size_t)min(qb + j, R - 1) * LPR];      // rows past R repeat the last one
      Piece<T>::unpack(raw, qf[j]);
    }
    float m[kQB], l[kQB], acc[kQB][EPL];
#pragma unroll
    for (int j = 0; j < kQB; ++j) {
      m[j] = -INFINITY;
      l[j] = 0.f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) acc[j][i] = 0.f;
    }

    // kUnroll rows per lane group and trip, all their loads issued before the first use
    for (int tb = t0 + group; tb < t1; tb += GROUPS * kUnroll) {
      uint4 kraw[kUnroll], vraw[kUnroll];
      float cc[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int t = tb + u * GROUPS;
        const int tc = min(t, t1 - 1);
        kraw[u] = Kp[(size_t)tc * LPR];
        vraw[u] = Vp[(size_t)tc * LPR];
        cc[u] = cnt ? (float)cnt[tc] : 1.f;
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        if (tb + u * GROUPS >= t1) break;                        // uniform per lane group
        float kf[EPL], vf[EPL];
        Piece<T>::unpack(kraw[u], kf);
        Piece<T>::unpack(vraw[u], vf);
        const float c = cc[u];
#pragma unroll
        for (int j = 0; j < kQB; ++j) {
          float d = 0.f;
#pragma unroll
          for (int i = 0; i < EPL; ++i) d = fmaf(qf[j][i], kf[i], d);
          const float s = row_group_sum<LPR>(d) * sh.scale_log2;
          // online softmax; the running maximum rises only a few times per lane group, so the rescale of
          // the numerator stays out of the common path (the first row meets m = -inf: corr = 0)
          if (s > m[j]) {
            const float corr = __builtin_amdgcn_exp2f(m[j] - s);
            l[j] *= corr;
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[j][i] *= corr;
            m[j] = s;
          }
          const float p = __builtin_amdgcn_exp2f(s - m[j]);
          l[j] = fmaf(c, p, l[j]);                               // c copies of the slot in the denominator
#pragma unroll
          for (int i = 0; i < EPL; ++i) acc[j][i] = fmaf(p, vf[i], acc[j][i]);
        }
      }
    }

    // the lane groups of the workgroup, in group order
#pragma unroll
    for (int j = 0; j < kQB; ++j) {
#pragma unroll
      for (int i = 0; i < EPL; ++i) sm_acc[group][j][piece * EPL + i] = acc[j][i];
      if (piece == 0) sm_ml[group][j] = make_float2(m[j], l[j]);
    }
    __syncthreads();
    for (int o = tid; o < kQB * D; o += kThreads) {
      const int j = o / D, dch = o % D;
      if (qb + j < R) {
        float M = -INFINITY;
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) M = fmaxf(M, sm_ml[g][j].x);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
          const float2 ml = sm_ml[g][j];
          if (ml.y > 0.f) {                                      // a group that saw no row has m = -inf, l = 0
            const float w = __builtin_amdgcn_exp2f(ml.x - M);
            num = fmaf(sm_acc[g][j][dch], w, num);
            den = fmaf(ml.y, w, den);
          }
        }
        float* dst = part + part_index(un.index, chunk, R, qb + j, D);
        dst[dch] = num;
        if (dch == 0) { dst[D] = M; dst[D + 1] = den; }
      }
    }
    __syncthreads();
  }
}

// out[unit, row, :] from the unit's chunk partials, in chunk order.  One workgroup of D threads per (unit, row).
template <int D>
__global__ __launch_bounds__(D) void decode_reduce_kernel(const UnitTable tab, const Shape sh,
                                                          const float* __restrict__ part, float* __restrict__ out) {
  const int R = sh.R;
  const Unit un = tab.u[blockIdx.x / R];
  const int row = blockIdx.x % R;
  const int nc = dec_chunks(un.len);
  const int d = threadIdx.x;
  float M = -INFINITY;
  for (int c = 0; c < nc; ++c) M = fmaxf(M, part[part_index(un.index, c, R, row, D) + D]);
  float num = 0.f, den = 0.f;
  for (int c = 0; c < nc; ++c) {
    const float* src = part + part_index(un.index, c, R, row, D);
    if (src[D + 1] > 0.f) {
      const float w = __builtin_amdgcn_exp2f(src[D] - M);
      num = fmaf(src[d], w, num);
      den = fmaf(src[D + 1], w, den);
    }
  }
  out[((size_t)un.index * R + row) * D + d] = num / den;
}

template <typename T, int D>
hipError_t launch_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                    const int32_t* counts, float* part, float* out, hipStream_t stream) {
  int widest = 1;
  for (int i = 0; i < tab.n_units; ++i) widest = std::max(widest, dec_chunks(tab.u[i].len));
  hipLaunchKernelGGL((decode_partial_kernel<T, D>), dim3(widest, tab.n_units), dim3(kThreads), 0, stream, tab, sh,
                     (const T*)Q, (const T*)K, (const T*)V, counts, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((decode_reduce_kernel<D>), dim3(tab.n_units * sh.R), dim3(D), 0, stream, tab, sh, part, out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* Q, const void* K,
                         const void* V, const int32_t* counts, float* part, float* out, hipStream_t stream) {
  if (dt == KVS_F32) {
    return sh.D == 64 ? launch_t<float, 64>(tab, sh, Q, K, V, counts, part, out, stream)
                      : launch_t<float, 128>(tab, sh, Q, K, V, counts, part, out, stream);
  }
  return sh.D == 64 ? launch_t<uint16_t, 64>(tab, sh, Q, K, V, counts, part, out, stream)
                    : launch_t<uint16_t, 128>(tab, sh, Q, K, V, counts, part, out, stream);
}

}  // namespace kvs
