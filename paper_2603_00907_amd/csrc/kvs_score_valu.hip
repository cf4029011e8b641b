// Score kernels, vector-ALU path: any dtype, any number of query rows.
//
// Computes, per unit, the attention of every query row over all cached Keys (Sec. 4.1, Eq.
// attn_def_vec) in two sweeps over K: sweep 0 leaves the softmax statistics (running maximum and
// sum of exponentials, base-2 domain) of every token chunk; sweep 1 recomputes the logits,
// normalises them with the unit-wide statistics and averages over the query rows into alpha_bar.
// (o_bar is accumulated by a separate streaming pass over V, see kvs_select.hip.)
//
// Layout: a row of K is read by LPR = row_bytes / 16 adjacent lanes, 16 bytes each, so one
// wavefront load instruction fetches 64 / LPR whole rows.  Dot products are reduced across the
// LPR lanes with DPP adds.  This is the path for query windows of one to three rows and for units
// shorter than an MFMA tile; the matrix-core kernels live in kvs_score_mfma.hip.
#include "kvs_device.h"

namespace kvs {
namespace {

constexpr int kQB = 8;          // query rows held in registers at a time
constexpr int kThreads = 256;

template <typename T, int D, int PHASE>
__global__ __launch_bounds__(kThreads) void score_valu_kernel(
    const UnitTable tab, const Shape sh, const T* __restrict__ Q, const T* __restrict__ K,
    const int32_t* __restrict__ counts_in, float* __restrict__ alpha_bar, float2* __restrict__ stats_part,
    const float* __restrict__ c_row) {
  constexpr int EPL = Piece<T>::N;          // elements per lane
  constexpr int LPR = D / EPL;              // lanes per row
  constexpr int RPW = kWave / LPR;          // rows per wavefront load
  constexpr int RPB = RPW * (kThreads / kWave);

  __shared__ float2 sm_stats[(kThreads / kWave) * RPW][kQB];
  __shared__ float sm_c[KVS_MAX_Q_ROWS];

  const int ui = find_unit(tab, blockIdx.x);
  const Unit un = tab.unit(ui);
  const int chunk = blockIdx.x - un.chunk_base;
  const int t0 = chunk * un.chunk_len;
  const int t1 = min(un.len, t0 + un.chunk_len);
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int grp = lane / LPR, piece = lane % LPR;
  const int R = sh.R;
  const size_t part_base = ((size_t)un.index * kMaxChunks);

  const uint4* Kp = reinterpret_cast<const uint4*>(K + (size_t)un.in_row * D) + piece;
  const uint4* Qp = reinterpret_cast<const uint4*>(Q + (size_t)un.index * R * D) + piece;

  if (PHASE == 1) load_row_consts(c_row, un.index, R, sm_c);

  for (int qb = 0; qb < R; qb += kQB) {
    float qf[kQB][EPL];
    float cq[kQB];
    int lim[kQB];                              // causal window: the last row query qb + j attends to
#pragma unroll
    for (int j = 0; j < kQB; ++j) {
      lim[j] = last_seen_row(sh.causal, un.len, qb + j);
      if (qb + j < R) {
        const uint4 raw = Qp[(size_t)(qb + j) * LPR];
        Piece<T>::unpack(raw, qf[j]);
        cq[j] = (PHASE == 1) ? sm_c[qb + j] : 0.f;
      } else {
#pragma unroll
        for (int i = 0; i < EPL; ++i) qf[j][i] = 0.f;
        cq[j] = INFINITY;                      // exp2(-inf) = 0: a padding row adds nothing
      }
    }
    float m[kQB], l[kQB];
#pragma unroll
    for (int j = 0; j < kQB; ++j) { m[j] = -INFINITY; l[j] = 0.f; }

    // kUnroll rows of a lane group are requested before the first is used (one row per trip left the sweep
    // waiting for memory most of the time)
    constexpr int kUnroll = 4;
    for (int tb = t0 + wave * RPW + grp; tb < t1; tb += RPB * kUnroll) {
      uint4 raw[kUnroll];
      int cn[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int tc = min(tb + u * RPB, t1 - 1);
        raw[u] = Kp[(size_t)tc * LPR];
        cn[u] = counts_in ? counts_in[un.in_row + tc] : 1;
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int t = tb + u * RPB;
        if (t >= t1) break;
        float kf[EPL];
        Piece<T>::unpack(raw[u], kf);
        // a row that stands for c tokens with this Key: c equal softmax terms, i.e. the logit plus log c
        const float lc = counts_in ? log2f((float)cn[u]) : 0.f;
        float a = 0.f;
#pragma unroll
        for (int j = 0; j < kQB; ++j) {
          if (qb + j >= R) break;                  // uniform: the last block of rows may be a short one
          float d = 0.f;
#pragma unroll
          for (int i = 0; i < EPL; ++i) d = fmaf(qf[j][i], kf[i], d);
          const float s = fmaf(row_group_sum<LPR>(d), sh.scale_log2, lc);
          if (t > lim[j]) continue;              // masked: no term in this row's softmax
          if (PHASE == 0) {
            if (s > m[j]) {
              l[j] = l[j] * __builtin_amdgcn_exp2f(m[j] - s) + 1.f;
              m[j] = s;
            } else {
              l[j] += __builtin_amdgcn_exp2f(s - m[j]);
            }
          } else {
            a += __builtin_amdgcn_exp2f(s - cq[j]);
          }
        }
        if (PHASE == 1 && piece == 0) {
          // the lane that owns the row keeps its running sum over the blocks of query rows
          if (qb != 0) a += alpha_bar[un.in_row + t];
          alpha_bar[un.in_row + t] = a;
        }
      }
    }

    if (PHASE == 0) {
      if (piece == 0) {
#pragma unroll
        for (int j = 0; j < kQB; ++j) sm_stats[wave * RPW + grp][j] = make_float2(m[j], l[j]);
      }
      __syncthreads();
      if (tid < kQB && qb + tid < R) {
        float M = -INFINITY;
        for (int g = 0; g < RPB; ++g) M = fmaxf(M, sm_stats[g][tid].x);
        float Z = 0.f;
        for (int g = 0; g < RPB; ++g) {
          const float2 s = sm_stats[g][tid];
          if (s.y > 0.f) Z += s.y * __builtin_amdgcn_exp2f(s.x - M);
        }
        stats_part[(part_base + chunk) * R + qb + tid] = make_float2(M, Z);
      }
      __syncthreads();
    }
  }
}

// Unit-wide softmax statistics of every query row from the chunks' (max, sum) pairs, as the one
// constant sweep 1 needs: c[q] = M_q + log2(Z_q * R), so that alpha[q,t] / R = exp2(logit2 - c[q]).
// One workgroup per unit: every sweep-1 workgroup needs all of c, and 64 chunks x R pairs fetched
// and reduced by each of them cost a fifth of that sweep.  Two threads share a row and take half of
// the chunks each, all their loads in flight at once (a loop with a run-time trip count would
// serialise the round trips); the order of the additions is fixed.
__global__ __launch_bounds__(kThreads) void score_finalize_kernel(const UnitTable tab, const Shape sh,
                                                                  const float2* __restrict__ stats_part,
                                                                  float* __restrict__ c_row,
                                                                  unsigned int* __restrict__ sel_shared) {
  constexpr int HALF = kMaxChunks / 2;
  // the exchange area of the selection that follows starts from zero (it has kInlineUnits entries: larger groups
  // do not use it)
  if (sel_shared != nullptr && blockIdx.x < kInlineUnits) {
    uint4* z = reinterpret_cast<uint4*>(sel_shared + (size_t)blockIdx.x * kSelSharedInts);
    for (int i = threadIdx.x; i < kSelSharedInts / 4; i += kThreads) z[i] = make_uint4(0u, 0u, 0u, 0u);
  }
  __shared__ float2 sm_pair[2][128];
  const Unit un = tab.unit(blockIdx.x);
  const int R = sh.R;
  const size_t part_base = (size_t)un.index * kMaxChunks;
  const int tid = threadIdx.x;
  const int h = tid / 128, r = tid % 128;
  for (int q0 = 0; q0 < R; q0 += 128) {
    const int q = q0 + r;
    float2 v[HALF];
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      const int c = h * HALF + i;
      v[i] = make_float2(-INFINITY, 0.f);
      if (q < R && c < un.n_chunks) v[i] = stats_part[(part_base + c) * R + q];
    }
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < HALF; ++i) M = fmaxf(M, v[i].x);
    float Z = 0.f;
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      if (v[i].y > 0.f) Z += v[i].y * __builtin_amdgcn_exp2f(v[i].x - M);
    }
    sm_pair[h][r] = make_float2(M, Z);
    __syncthreads();
    if (h == 0 && q < R) {
      const float2 a = sm_pair[0][r], b = sm_pair[1][r];
      const float Mq = fmaxf(a.x, b.x);
      float Zq = a.y * __builtin_amdgcn_exp2f(a.x - Mq);
      if (b.y > 0.f) Zq += b.y * __builtin_amdgcn_exp2f(b.x - Mq);
      c_row[(size_t)un.index * R + q] = Mq + log2f(Zq * (float)R);
    }
    __syncthreads();
  }
}

}  // namespace

hipError_t launch_score_finalize(const UnitTable& tab, const Shape& sh, const Workspace& ws, hipStream_t stream) {
  hipLaunchKernelGGL(score_finalize_kernel, dim3(tab.n_units), dim3(kThreads), 0, stream, tab, sh, ws.stats_part,
                     ws.c_row, ws.sel_shared);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_score_valu_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                                      const int32_t* counts_in, float* alpha_bar, const Workspace& ws,
                                      hipStream_t stream) {
  dim3 grid(tab.total_chunks), block(kThreads);
  hipLaunchKernelGGL((score_valu_kernel<T, D, 0>), grid, block, 0, stream, tab, sh, (const T*)Q, (const T*)K,
                     counts_in, alpha_bar, ws.stats_part, ws.c_row);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if ((e = launch_score_finalize(tab, sh, ws, stream)) != hipSuccess) return e;
  hipLaunchKernelGGL((score_valu_kernel<T, D, 1>), grid, block, 0, stream, tab, sh, (const T*)Q, (const T*)K,
                     counts_in, alpha_bar, ws.stats_part, ws.c_row);
  return hipGetLastError();
}

hipError_t launch_score_valu(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* Q, const void* K,
                             const int32_t* counts_in, float* alpha_bar, const Workspace& ws, hipStream_t stream) {
  if (dt == KVS_F32) {
    return sh.D == 64 ? launch_score_valu_t<float, 64>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream)
                      : launch_score_valu_t<float, 128>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream);
  }
  return sh.D == 64 ? launch_score_valu_t<uint16_t, 64>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream)
                    : launch_score_valu_t<uint16_t, 128>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream);
}

}  // namespace kvs
