// Merge-and-compact kernel: one pass over K and V.
//
// For every output slot S (a run of consecutive tokens t0..t1 chained by selected edges):
//   r_t = V[t] - o_bar
//   A_t = alpha_t |1 - 2 alpha_t| ||r_t||          (= ||c_tt||,      Sec. 4.2, Eqs. c11_def, c22_def)
//   C_t = alpha_t alpha_{t+1} ||r_t + r_{t+1}||    (= ||c_{t,t+1}||, Eq. c12_def), inner edges only
//   u_t = A_t - C_{t-1} - C_t
//   K_out[S] = sum u_t K[t] / sum u_t              (Eq. kstar_final for a pair; the same weight form
//                                                    for a longer run), arithmetic mean of the run if
//                                                    the denominator is not positive and finite
//   V_out[S] = sum V[t]                            (Sec. 3.1), counts[S] = t1 - t0 + 1
// A slot of one token is copied bit for bit.
//
// Layout: a row is read by LPR = row_bytes / 16 adjacent lanes (16 bytes each); such a lane group
// walks a contiguous range of kMergeTokens / groups tokens in order, carrying the open slot's
// accumulators in registers.  A group starts at the first slot that begins inside its range and
// runs past the range's end until that last slot is closed, so every slot is summed by exactly
// one group, in token order: the result does not depend on the launch geometry and needs neither
// atomics nor a carry between workgroups.  The next token's rows are requested before the current
// token is processed.
#include "kvs_device.h"

namespace kvs {
namespace {

constexpr int kThreads = 256;

template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
#pragma unroll
  for (int off = LPR / 2; off >= 1; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void merge_kernel(
    const UnitTable tab, const Shape sh, const T* __restrict__ K, const T* __restrict__ V,
    const float* __restrict__ alpha_bar, const float* __restrict__ o_bar, const uint8_t* __restrict__ edge_mask,
    const int32_t* __restrict__ slot, T* __restrict__ K_out, T* __restrict__ V_out, int32_t* __restrict__ counts) {
  constexpr int EPL = Piece<T>::N;
  constexpr int LPR = D / EPL;
  constexpr int GROUPS = kThreads / LPR;
  constexpr int TPG = kMergeTokens / GROUPS;

  // which unit: merge workgroups are numbered by m_base
  int ui = 0;
  while (ui + 1 < tab.n_units && tab.u[ui + 1].m_base <= (int)blockIdx.x) ++ui;
  const Unit un = tab.u[ui];
  const int n = un.len;
  const int tid = threadIdx.x;
  const int group = tid / LPR, piece = tid % LPR;
  const int a = ((int)blockIdx.x - un.m_base) * kMergeTokens + group * TPG;   // nominal range [a, b)
  const int b = min(n, a + TPG);
  if (a >= n) return;

  const uint4* Kp = reinterpret_cast<const uint4*>(K + (size_t)un.in_row * D) + piece;
  const uint4* Vp = reinterpret_cast<const uint4*>(V + (size_t)un.in_row * D) + piece;
  uint4* Ko = reinterpret_cast<uint4*>(K_out + (size_t)un.out_row * D) + piece;
  uint4* Vo = reinterpret_cast<uint4*>(V_out + (size_t)un.out_row * D) + piece;
  int32_t* cnt = counts + un.out_row;
  const float* al = alpha_bar + un.in_row;
  const uint8_t* mk = edge_mask + un.in_row;
  const int32_t* sl = slot + un.in_row;

  float o[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) o[i] = o_bar[(size_t)un.index * D + piece * EPL + i];

  // first slot that begins inside [a, b)
  int t = a;
  while (t < b && t > 0 && mk[t - 1]) ++t;
  if (t >= b) return;

  float accK[EPL], accV[EPL], kprev[EPL], rprev[EPL];
  float U = 0.f, pend = 0.f, aprev = 0.f;
  int run = 0, out_slot = 0;

  uint4 kraw = Kp[(size_t)t * LPR], vraw = Vp[(size_t)t * LPR];
  float alpha_t = al[t];
  int mask_t = mk[t];

  while (true) {
    // request the next token before working on this one (clamped: the last request is discarded)
    const int tn = min(t + 1, n - 1);
    const uint4 kraw_n = Kp[(size_t)tn * LPR], vraw_n = Vp[(size_t)tn * LPR];
    const float alpha_n = al[tn];
    const int mask_n = mk[tn];

    if (run == 0 && mask_t == 0) {
      const int s = sl[t];
      if ((unsigned)s < (unsigned)un.n_out) {      // a slot map from outside the library is not trusted
        Ko[(size_t)s * LPR] = kraw;
        Vo[(size_t)s * LPR] = vraw;
        if (piece == 0) cnt[s] = 1;
      }
    } else {
      float kf[EPL], vf[EPL], rr[EPL];
      Piece<T>::unpack(kraw, kf);
      Piece<T>::unpack(vraw, vf);
      float ss = 0.f, sc = 0.f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        rr[i] = vf[i] - o[i];
        ss = fmaf(rr[i], rr[i], ss);
      }
      if (run > 0) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
          const float p = rprev[i] + rr[i];
          sc = fmaf(p, p, sc);
        }
      }
      ss = group_sum<LPR>(ss);
      sc = group_sum<LPR>(sc);
      const float A = alpha_t * fabsf(1.f - 2.f * alpha_t) * sqrtf(ss);
      if (run == 0) {
        out_slot = sl[t];
        U = 0.f;
        pend = A;
#pragma unroll
        for (int i = 0; i < EPL; ++i) { accK[i] = 0.f; accV[i] = vf[i]; }
      } else {
        const float C = aprev * alpha_t * sqrtf(sc);
        const float u_prev = pend - C;
        U += u_prev;
        pend = A - C;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
          accK[i] = fmaf(u_prev, kprev[i], accK[i]);
          accV[i] += vf[i];
        }
      }
      ++run;
      if (mask_t == 0) {               // the slot ends here
        U += pend;
#pragma unroll
        for (int i = 0; i < EPL; ++i) accK[i] = fmaf(pend, kf[i], accK[i]);
        float outk[EPL];
        if (U > 0.f && U < INFINITY) {
          const float inv = 1.f / U;
#pragma unroll
          for (int i = 0; i < EPL; ++i) outk[i] = accK[i] * inv;
        } else {                       // no usable weights: arithmetic mean of the run
#pragma unroll
          for (int i = 0; i < EPL; ++i) outk[i] = 0.f;
          for (int j = t - run + 1; j <= t; ++j) {
            float kj[EPL];
            Piece<T>::unpack(Kp[(size_t)j * LPR], kj);
#pragma unroll
            for (int i = 0; i < EPL; ++i) outk[i] += kj[i];
          }
          const float inv = 1.f / (float)run;
#pragma unroll
          for (int i = 0; i < EPL; ++i) outk[i] *= inv;
        }
        if ((unsigned)out_slot < (unsigned)un.n_out) {
          Ko[(size_t)out_slot * LPR] = Piece<T>::pack(outk);
          Vo[(size_t)out_slot * LPR] = Piece<T>::pack(accV);
          if (piece == 0) cnt[out_slot] = run;
        }
        run = 0;
      } else {
        aprev = alpha_t;
#pragma unroll
        for (int i = 0; i < EPL; ++i) { kprev[i] = kf[i]; rprev[i] = rr[i]; }
      }
    }

    const bool slot_closed = (mask_t == 0);
    ++t;
    if (t >= n || (t >= b && slot_closed)) break;
    kraw = kraw_n; vraw = vraw_n; alpha_t = alpha_n; mask_t = mask_n;
  }
}

}  // namespace

template <typename T, int D>
static hipError_t launch_merge_t(const UnitTable& tab, const Shape& sh, const void* K, const void* V,
                                 const float* alpha_bar, const float* o_bar, const uint8_t* edge_mask,
                                 const int32_t* slot, void* K_out, void* V_out, int32_t* counts,
                                 hipStream_t stream) {
  hipLaunchKernelGGL((merge_kernel<T, D>), dim3(tab.total_mblocks), dim3(kThreads), 0, stream, tab, sh,
                     (const T*)K, (const T*)V, alpha_bar, o_bar, edge_mask, slot, (T*)K_out, (T*)V_out, counts);
  return hipGetLastError();
}

hipError_t launch_merge(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* K, const void* V,
                        const float* alpha_bar, const float* o_bar, const uint8_t* edge_mask,
                        const int32_t* slot, void* K_out, void* V_out, int32_t* counts, hipStream_t stream) {
  if (dt == KVS_F32) {
    return sh.D == 64
               ? launch_merge_t<float, 64>(tab, sh, K, V, alpha_bar, o_bar, edge_mask, slot, K_out, V_out, counts, stream)
               : launch_merge_t<float, 128>(tab, sh, K, V, alpha_bar, o_bar, edge_mask, slot, K_out, V_out, counts, stream);
  }
  return sh.D == 64
             ? launch_merge_t<uint16_t, 64>(tab, sh, K, V, alpha_bar, o_bar, edge_mask, slot, K_out, V_out, counts, stream)
             : launch_merge_t<uint16_t, 128>(tab, sh, K, V, alpha_bar, o_bar, edge_mask, slot, K_out, V_out, counts, stream);
}

}  // namespace kvs
