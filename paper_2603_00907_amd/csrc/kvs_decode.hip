// Decode attention over a merged cache (the consumer of kvs_merge_compact's outputs).
//
// A row (k', V', c) of a merged cache stands for c tokens that all carry the Key k' and whose Values
// add up to V' (Sec. 3.1: the pair (k_m, k_{m+1}) is replaced by (k, k), the Values are summed, and the
// cardinality is carried along).  Attention of a query q over such a cache is
//   o = sum_S exp(e_S) V'_S / sum_S c_S exp(e_S),      e_S = scale * q . k'_S,
// i.e. ordinary attention over the c_S copies of every slot.  With c = 1 it is plain attention.
//
// Split over the rows of a unit (chunks of at least 256 rows, at most 64 per unit, one workgroup
// each; the grid is chunks x units): LPR adjacent lanes read one K row and one V row (16 bytes each), four query rows at a time
// sit in registers, every lane group keeps an online softmax (running maximum, denominator,
// D-wide numerator) for its rows, the groups of a workgroup are combined through LDS, and a second
// small kernel combines the chunks.  Everything is ordered: no atomics, results do not depend on
// timing.  The kernel is meant for decode-sized query blocks (at most KVS_MAX_DECODE_ROWS rows per
// unit); it reads the cache once per block of four query rows.
//
// bf16 caches whose units have at least 32 rows take decode_mfma_kernel instead: both products on
// v_mfma_f32_32x32x16_bf16, 32 query rows per pass, the operands loaded from memory in the MFMA layout (a lane
// fetches the 16-byte pieces of ITS row), so nothing is staged in LDS and the wavefronts of a workgroup, which
// split the chunk's 32-row tiles, never wait for each other inside the loop.  The chunk partials have the same
// format and go through the same second kernel.
#include <algorithm>
#include <cstdlib>
#include <cstring>

#include "kvs_device.h"

namespace kvs {
namespace {

#ifndef KVS_DEC_THREADS
#define KVS_DEC_THREADS 256
#endif
constexpr int kThreads = KVS_DEC_THREADS;
constexpr int kQB = 4;                    // query rows per block
#ifndef KVS_DEC_UNROLL
#define KVS_DEC_UNROLL 2
#endif
constexpr int kUnroll = KVS_DEC_UNROLL;   // cache rows per lane group in flight
#ifndef KVS_DEC_CHUNK
#define KVS_DEC_CHUNK 256
#endif
constexpr int kDecMinChunk = KVS_DEC_CHUNK;   // rows per workgroup, at least

constexpr int kDecMaxMinChunk = 1024;
constexpr int kDecWorkgroups = 2048;          // workgroups a launch aims for (8 per CU)

// Chunking of a unit's rows: a function of its length and of the launch's least chunk length.
__host__ __device__ inline int dec_chunk_len(int len, int min_chunk) {
  const int per = (len + kMaxChunks - 1) / kMaxChunks;
  const int rounded = (per + kWave - 1) / kWave * kWave;
  return rounded > min_chunk ? rounded : min_chunk;
}
__host__ __device__ inline int dec_chunks(int len, int min_chunk) {
  const int cl = dec_chunk_len(len, min_chunk);
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

  const Unit un = tab.unit(blockIdx.y);
  const int chunk = blockIdx.x;
  if (chunk >= dec_chunks(un.len, sh.dec_chunk)) return;               // the grid is as wide as the longest unit needs
  const int clen = dec_chunk_len(un.len, sh.dec_chunk);
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
  const Unit un = tab.unit(blockIdx.x / R);
  const int row = blockIdx.x % R;
  const int nc = dec_chunks(un.len, sh.dec_chunk);
  const int d = threadIdx.x;
  // the maximum over the chunks first (all loads in flight at once), then the weighted sums in chunk order,
  // eight chunks' loads in flight at a time: the partials come from memory and a loop that waits for every
  // load costs a round trip per chunk
  float M = -INFINITY;
  {
    float mv[kMaxChunks / 8];
    for (int c0 = 0; c0 < nc; c0 += kMaxChunks / 8) {
#pragma unroll
      for (int i = 0; i < kMaxChunks / 8; ++i) mv[i] = part[part_index(un.index, min(c0 + i, nc - 1), R, row, D) + D];
#pragma unroll
      for (int i = 0; i < kMaxChunks / 8; ++i) M = fmaxf(M, mv[i]);
    }
  }
  float num = 0.f, den = 0.f;
  for (int c0 = 0; c0 < nc; c0 += 8) {
    float x[8], m[8], l[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float* src = part + part_index(un.index, min(c0 + i, nc - 1), R, row, D);
      x[i] = src[d];
      m[i] = src[D];
      l[i] = src[D + 1];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (c0 + i < nc && l[i] > 0.f) {
        const float w = __builtin_amdgcn_exp2f(m[i] - M);
        num = fmaf(x[i], w, num);
        den = fmaf(l[i], w, den);
      }
    }
  }
  out[((size_t)un.index * R + row) * D + d] = num / den;
}

// ------------------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ bf16x8 pack8(const float* f) {
  return as_bf16x8(make_uint4(cvt_pk_bf16(f[0], f[1]), cvt_pk_bf16(f[2], f[3]), cvt_pk_bf16(f[4], f[5]),
                              cvt_pk_bf16(f[6], f[7])));
}
// eight floats -> hi + lo: hi = bf16(f), lo = bf16(f - hi)
__device__ __forceinline__ void split8(const float* f, bf16x8& hi, bf16x8& lo) {
  uint32_t h[4];
  float r[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    h[i] = cvt_pk_bf16(f[2 * i], f[2 * i + 1]);
    r[2 * i] = f[2 * i] - bf16_lo(h[i]);
    r[2 * i + 1] = f[2 * i + 1] - bf16_hi(h[i]);
  }
  hi = as_bf16x8(make_uint4(h[0], h[1], h[2], h[3]));
  lo = pack8(r);
}

constexpr int kMfmaThreads = 256;
constexpr int kMfmaWaves = kMfmaThreads / kWave;
constexpr int kTile = 32;

// Per tile of 32 cache rows and block of 32 query rows (one per lane column):
//   S[t, q] = K_tile Q^T               8 (D = 128) products; a lane holds one query column and 16 rows
//   online softmax per column          the running maximum is lane-private (exchanged once between the halves of
//                                      the wavefront); the numerator is rescaled only when the maximum rises
//   Y = V_tile[:, 32 db ..] I          the V block in the accumulator layout, which is the token-major operand
//                                      layout the next product needs (exact: bf16 times one)
//   O^T[d, q] += Y^T P                 P as a bf16 pair hi + lo
template <int D>
__global__ __launch_bounds__(kMfmaThreads, 2) void decode_mfma_kernel(
    const UnitTable tab, const Shape sh, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, const int32_t* __restrict__ counts, float* __restrict__ part) {
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int ROWB = D * 2;
  constexpr int ACCW = D + 4;               // numerator, maximum, denominator; rows stay 16-byte aligned
  __shared__ __attribute__((aligned(16))) float sm_acc[kMfmaWaves][kTile][ACCW];
  __shared__ __attribute__((aligned(16))) float sm_cnt[kMfmaWaves][kTile];

  const Unit un = tab.unit(blockIdx.y);
  const int chunk = blockIdx.x;
  if (chunk >= dec_chunks(un.len, sh.dec_chunk)) return;               // the grid is as wide as the longest unit needs
  const int clen = dec_chunk_len(un.len, sh.dec_chunk);
  const int t0 = chunk * clen;
  const int t1 = min(un.len, t0 + clen);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int col = lane % 32, half = lane / 32;
  const int R = sh.R;
  const float sl2 = sh.scale_log2;
  const unsigned char* Kg = reinterpret_cast<const unsigned char*>(K + (size_t)un.in_row * D);
  const unsigned char* Vg = reinterpret_cast<const unsigned char*>(V + (size_t)un.in_row * D);
  const uint16_t* Qu = Q + (size_t)un.index * R * D;
  const int32_t* cnt = counts ? counts + un.in_row : nullptr;

  // identity operand: element i of k-step kk is 1 where 16 kk + 8 half + i is this lane's column
  bf16x8 ident[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k0 = 16 * kk + 8 * half + 2 * i;
      w[i] = (k0 == col ? 0x3F80u : 0u) | (k0 + 1 == col ? 0x3F800000u : 0u);
    }
    ident[kk] = as_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
  }
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  for (int qb = 0; qb < R; qb += kTile) {
    const int qrow = qb + col;
    bf16x8 bq[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (qrow < R) raw = *reinterpret_cast<const uint4*>(Qu + (size_t)qrow * D + kk * 16 + 8 * half);
      bq[kk] = as_bf16x8(raw);
    }
    f32x16 accO[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) accO[db] = zero;
    float m_run = -INFINITY, l_run = 0.f;

    for (int j = wave; j < ntiles; j += kMfmaWaves) {
      // the ragged last tile is moved back to end at the chunk's end (every unit on this path has at least 32
      // rows); the `shift` rows it shares with the tile before drop out
      const int tile_t0 = t0 + j * kTile;
      const int base_t = min(tile_t0, t1 - kTile);
      const int shift = tile_t0 - base_t;
      // operands straight from memory: this lane's row of the tile, 16 bytes per k-step
      const unsigned char* krow = Kg + (size_t)(base_t + col) * ROWB + half * 16;
      const unsigned char* vrow = Vg + (size_t)(base_t + col) * ROWB + half * 16;
      bf16x8 ka[KS], va[KS];
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) ka[kk] = as_bf16x8(*reinterpret_cast<const uint4*>(krow + kk * 32));
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) va[kk] = as_bf16x8(*reinterpret_cast<const uint4*>(vrow + kk * 32));
      if (cnt != nullptr && half == 0) sm_cnt[wave][col] = (float)cnt[base_t + col];

      f32x16 acc = zero;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], bq[kk], acc, 0, 0, 0);
      // accumulator element v: cache row 8 (v / 4) + 4 half + v % 4 of the tile, query column `col`
      float sv[16];
      float tm = -INFINITY;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = 8 * (v / 4) + 4 * half + (v % 4);
        sv[v] = (row >= shift) ? acc[v] * sl2 : -INFINITY;
        tm = fmaxf(tm, sv[v]);
      }
      tm = fmaxf(tm, __shfl_xor(tm, 32, kWave));           // both halves feed the same column of O^T
      if (tm > m_run) {                                    // rare after the first tiles
        const float corr = __builtin_amdgcn_exp2f(m_run - tm);     // the first tile meets -inf: corr = 0
        l_run *= corr;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
          for (int v = 0; v < 16; ++v) accO[db][v] *= corr;
        }
        m_run = tm;
      }
      float p[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) p[v] = __builtin_amdgcn_exp2f(sv[v] - m_run);
      // denominator: c copies of every slot
      if (cnt != nullptr) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 c4 = *reinterpret_cast<const float4*>(&sm_cnt[wave][8 * g + 4 * half]);
          l_run = fmaf(c4.x, p[4 * g], l_run);
          l_run = fmaf(c4.y, p[4 * g + 1], l_run);
          l_run = fmaf(c4.z, p[4 * g + 2], l_run);
          l_run = fmaf(c4.w, p[4 * g + 3], l_run);
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) l_run += p[v];
      }
      // as the operand of the next product, element i of k-step s is accumulator element 8 s + i
      bf16x8 ph[2], pl[2];
      split8(p, ph[0], pl[0]);
      split8(p + 8, ph[1], pl[1]);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        f32x16 y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[2 * db], ident[0], zero, 0, 0, 0);
        y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[2 * db + 1], ident[1], y, 0, 0, 0);
        float yf[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) yf[v] = y[v];
        const bf16x8 vt0 = pack8(yf), vt1 = pack8(yf + 8);     // exact: the values are bf16 numbers
        accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt0, ph[0], accO[db], 0, 0, 0);
        accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt1, ph[1], accO[db], 0, 0, 0);
        accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt0, pl[0], accO[db], 0, 0, 0);
        accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt1, pl[1], accO[db], 0, 0, 0);
      }
    }

    // the wavefronts of the workgroup, in wavefront order.  O^T element v of block db: channel
    // 32 db + 8 (v / 4) + 4 half + v % 4 of query column `col`
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        *reinterpret_cast<float4*>(&sm_acc[wave][col][32 * db + 8 * g + 4 * half]) =
            make_float4(accO[db][4 * g], accO[db][4 * g + 1], accO[db][4 * g + 2], accO[db][4 * g + 3]);
      }
    }
    if (half == 0) { sm_acc[wave][col][D] = m_run; sm_acc[wave][col][D + 1] = l_tot; }
    __syncthreads();
    for (int o = tid; o < kTile * D; o += kMfmaThreads) {
      const int q = o / D, dch = o % D;
      if (qb + q < R) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kMfmaWaves; ++w) M = fmaxf(M, sm_acc[w][q][D]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < kMfmaWaves; ++w) {
          const float lw = sm_acc[w][q][D + 1];
          if (lw > 0.f) {                                    // a wavefront that had no tile has m = -inf, l = 0
            const float wgt = __builtin_amdgcn_exp2f(sm_acc[w][q][D] - M);
            num = fmaf(sm_acc[w][q][dch], wgt, num);
            den = fmaf(lw, wgt, den);
          }
        }
        float* dst = part + part_index(un.index, chunk, R, qb + q, D);
        dst[dch] = num;
        if (dch == 0) { dst[D] = M; dst[D + 1] = den; }
      }
    }
    __syncthreads();
  }
}

template <int D>
hipError_t launch_mfma(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                       const int32_t* counts, float* part, float* out, hipStream_t stream) {
  int widest = 1;
  for (int i = 0; i < tab.n_units; ++i) widest = std::max(widest, dec_chunks(tab.unit(i).len, sh.dec_chunk));
  hipLaunchKernelGGL((decode_mfma_kernel<D>), dim3(widest, tab.n_units), dim3(kMfmaThreads), 0, stream, tab, sh,
                     (const uint16_t*)Q, (const uint16_t*)K, (const uint16_t*)V, counts, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((decode_reduce_kernel<D>), dim3(tab.n_units * sh.R), dim3(D), 0, stream, tab, sh, part, out);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                    const int32_t* counts, float* part, float* out, hipStream_t stream) {
  int widest = 1;
  for (int i = 0; i < tab.n_units; ++i) widest = std::max(widest, dec_chunks(tab.unit(i).len, sh.dec_chunk));
  hipLaunchKernelGGL((decode_partial_kernel<T, D>), dim3(widest, tab.n_units), dim3(kThreads), 0, stream, tab, sh,
                     (const T*)Q, (const T*)K, (const T*)V, counts, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((decode_reduce_kernel<D>), dim3(tab.n_units * sh.R), dim3(D), 0, stream, tab, sh, part, out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const UnitTable& tab, const Shape& sh_in, kvs_dtype dt, const void* Q, const void* K,
                         const void* V, const int32_t* counts, float* part, float* out, hipStream_t stream) {
  // Rows per workgroup: kDecMinChunk where the launch is small (a workgroup per 256 rows keeps every CU busy), more
  // where that would make many more workgroups than the chip holds at once (256 caches of 4096 rows: chunks of 512
  // rows take 0.120 ms against 0.128 with 256 and 0.149 with 128).
  Shape sh = sh_in;
  long long rows = 0;
  for (int i = 0; i < tab.n_units; ++i) rows += tab.unit(i).len;
  long long chunk = (rows / kDecWorkgroups + kWave - 1) / kWave * kWave;
  sh.dec_chunk = (int)(chunk < kDecMinChunk ? kDecMinChunk : chunk > kDecMaxMinChunk ? kDecMaxMinChunk : chunk);
  if (dt == KVS_F32) {
    return sh.D == 64 ? launch_t<float, 64>(tab, sh, Q, K, V, counts, part, out, stream)
                      : launch_t<float, 128>(tab, sh, Q, K, V, counts, part, out, stream);
  }
  // The vector-ALU kernel reads the cache once per four query rows: up to four rows it is as fast as the MFMA
  // kernel (both are latency-bound on caches of a few thousand rows), above that the MFMA kernel wins (measured,
  // 64 caches of 4096 rows: 42 against 62 us at 8 rows, 55 against 200 us at 32 rows).
  // KVS_DEBUG_DECODE_PATH forces one of them (used by the tests to cover both).
  const int force = debug_switch(KVS_DEBUG_DECODE_PATH);
  bool mfma = sh.R > kQB;
  if (force == 1) mfma = false;
  if (force == 2) mfma = true;
  for (int i = 0; i < tab.n_units; ++i) mfma = mfma && tab.unit(i).len >= kTile;   // its tiles hold 32 whole rows
  if (mfma) {
    return sh.D == 64 ? launch_mfma<64>(tab, sh, Q, K, V, counts, part, out, stream)
                      : launch_mfma<128>(tab, sh, Q, K, V, counts, part, out, stream);
  }
  return sh.D == 64 ? launch_t<uint16_t, 64>(tab, sh, Q, K, V, counts, part, out, stream)
                    : launch_t<uint16_t, 128>(tab, sh, Q, K, V, counts, part, out, stream);
}

}  // namespace kvs
