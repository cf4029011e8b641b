// Per-query aggregation of the sensitivity norms (bf16 inputs).
//
// Sec. 4 derives the forward-only vectors c_tt = alpha_t (1 - 2 alpha_t)(v_t - o) and
// c_{t,t+1} = -alpha_t alpha_{t+1} (v_t + v_{t+1} - 2o) (Eqs. c11_def-c12_def) for ONE query.  Here every
// query row q of the window keeps its own attention alpha^{(q)} and its own output o^{(q)} (Eq.
// attn_def_vec), and the NORMS are averaged over the R rows:
//   A_t = (1/R) sum_q alpha_t^{(q)} |1 - 2 alpha_t^{(q)}| ||v_t - o^{(q)}||
//   C_t = (1/R) sum_q alpha_t^{(q)} alpha_{t+1}^{(q)} ||v_t + v_{t+1} - 2 o^{(q)}||
// The merge kernel then uses A and C in the weight form of Eq. kstar_final.
//
// Four kernels after the two score sweeps (which leave the normaliser c[q] of every row):
//   pq_out_kernel         O^T[d, q] = sum_t V[t, d] P[t, q], P = alpha / R recomputed from K Q^T tile by tile.
//                         Both products run on v_mfma_f32_32x32x16_bf16.  The contraction over tokens needs
//                         V with the token index along the MFMA k dimension; a 32x32 block of the V tile is
//                         turned by one more MFMA against an identity operand (exact in bf16), which leaves it
//                         in the accumulator layout that IS the k-major operand layout of the next product
//                         (one block per wavefront, shared through LDS).
//                         P enters as a bf16 pair hi + lo, so that the rounding of P to bf16 does not limit
//                         the accuracy of o; the sum of the weights, as the pairs carry them, is kept beside it.
//                         Chunk partials go to memory and are added in chunk order.
//   pq_out_reduce_kernel  o^{(q)} = (sum of the chunk partials) / (sum of their weights): a convex combination of the
//                         Values with the weights as they were rounded, so that where a row puts nearly all its
//                         weight on one token, o - v_t is as accurate as the small weights of the others (dividing
//                         by the nominal sum 1 / R would leave the weights' rounding times ||v_t||).
//                         -2 o^{(q)} stored as a bf16 pair hi + lo, and ||o^{(q)}||^2.
//   pq_norms_kernel       per tile of 32 tokens: S' = Q K^T (logits), X' = (-2 O) V^T (hi and lo), then per (t, q)
//                         (accumulated on top of ||o||^2), then per (t, q)
//                         ||v_t - o||^2 = ||v_t||^2 + X',
//                         ||v_t + v_{t+1} - 2o||^2 = ||v_t + v_{t+1}||^2 + 2 (X'_t + X'_{t+1}),
//                         two square roots, and the sums over q.  Tiles overlap by one row (stride 31), so
//                         the next token of every output row is in the same tile.  Tokens where the expansions
//                         cancel (o^{(q)} close to v_t for some q) are marked.
//   pq_redo_kernel        the marked tokens once more, every squared norm as a sum of squared differences.
// COUNTS: the rows are slots of an already merged cache (Sec. 3.1, streaming regime), row t standing for c_t tokens
// whose Values add up to V[t]: every query row sees it as one token with logit e + ln c_t and value V[t] / c_t.  The
// products still run on the stored rows; log2 c_t joins the logit, and 1 / c_t scales the attention weight of the
// Value sum (o), the product V_t . o and the squared norms afterwards.
// A workgroup has four wavefronts; wavefront w owns query rows 32w .. 32w+31 of a pass of 128 rows and
// keeps their operands in registers; all four walk the same K and V tiles, staged through LDS (XOR-swizzled
// 16-byte pieces, as in the score kernels).  Results do not depend on timing: no atomics, fixed orders.
#include <type_traits>

#include "kvs_device.h"

namespace kvs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kTile = 32;                 // tokens per MFMA tile
constexpr int kPassRows = 32 * kWaves;    // query rows per pass over the chunk
constexpr int kRedoSpan = 4096;           // pq_redo: tokens per workgroup
constexpr float kCancel = 1.f / 16.f;     // pq_norms: a squared norm below this share of its leading term is formed again

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

// (one instruction; written out because the compiler forms it from nested fminf only now and then)
__device__ __forceinline__ float min3(float a, float b, float c) {
  float r;
  asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// c + a.lo * b.lo + a.hi * b.hi for two packed bf16 pairs (v_dot2c_f32_bf16)
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& u) { return __builtin_bit_cast(bf16x8, u); }

// eight floats -> bf16 operand (round to nearest even)
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

// The same, and w[i] = the value the pair stands for (hi + lo as floats).
__device__ __forceinline__ void split8w(const float* f, bf16x8& hi, bf16x8& lo, float* w) {
  uint32_t h[4], l[4];
  float r[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    h[i] = cvt_pk_bf16(f[2 * i], f[2 * i + 1]);
    r[2 * i] = f[2 * i] - bf16_lo(h[i]);
    r[2 * i + 1] = f[2 * i + 1] - bf16_hi(h[i]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    l[i] = cvt_pk_bf16(r[2 * i], r[2 * i + 1]);
    w[2 * i] = bf16_lo(h[i]) + bf16_lo(l[i]);
    w[2 * i + 1] = bf16_hi(h[i]) + bf16_hi(l[i]);
  }
  hi = as_bf16x8(make_uint4(h[0], h[1], h[2], h[3]));
  lo = as_bf16x8(make_uint4(l[0], l[1], l[2], l[3]));
}

// A 32-row tile of K or V: global -> registers -> LDS.  Piece p of row r lands in slot p ^ (r % LPR).
template <int D>
struct Tile {
  static constexpr int LPR = D / 8;                       // 16-byte pieces per row
  static constexpr int ROWB = D * 2;
  static constexpr int BYTES = kTile * ROWB;
  static constexpr int NP = kTile * LPR / kThreads;       // pieces per thread: 1 or 2
  // (two named registers instead of an array: an array handed on by reference across the loop stayed in
  // scratch memory, with a wait after every load)
  struct Regs { uint4 a, b; };
  __device__ __forceinline__ static Regs load(const unsigned char* tile_base, int tid) {
    Regs r;
    r.a = *reinterpret_cast<const uint4*>(tile_base + (size_t)tid * 16);
    r.b = (NP > 1) ? *reinterpret_cast<const uint4*>(tile_base + (size_t)(tid + kThreads) * 16) : make_uint4(0, 0, 0, 0);
    return r;
  }
  __device__ __forceinline__ static void store_piece(unsigned char* sm, const uint4& x, int pi) {
    const int row = pi / LPR, piece = pi % LPR;
    *reinterpret_cast<uint4*>(sm + row * ROWB + ((piece ^ (row % LPR)) * 16)) = x;
  }
  __device__ __forceinline__ static void store(unsigned char* sm, const Regs& r, int tid) {
    store_piece(sm, r.a, tid);
    if (NP > 1) store_piece(sm, r.b, tid + kThreads);
  }
  // MFMA operand of k-step kk for this lane: row `row`, elements 16 kk + 8 half .. + 7
  __device__ __forceinline__ static bf16x8 operand(const unsigned char* sm, int row, int kk, int half) {
    const int piece = 2 * kk + half;
    return *reinterpret_cast<const bf16x8*>(sm + row * ROWB + ((piece ^ (row % LPR)) * 16));
  }
  __device__ __forceinline__ static uint4 piece_at(const unsigned char* sm, int row, int piece) {
    return *reinterpret_cast<const uint4*>(sm + row * ROWB + ((piece ^ (row % LPR)) * 16));
  }
};

// Operand of k-step kk from a row-major [rows, D] bf16 matrix in memory (zero for a row that does not exist).
template <int D>
__device__ __forceinline__ bf16x8 row_operand(const uint16_t* __restrict__ m, int row, bool ok, int kk, int half) {
  uint4 raw = make_uint4(0, 0, 0, 0);
  if (ok) raw = *reinterpret_cast<const uint4*>(m + (size_t)row * D + kk * 16 + 8 * half);
  return as_bf16x8(raw);
}

// ------------------------------------------------------------------------------------------------
// o_part[(chunk of the launch), q, :] = sum over the chunk's tokens of (alpha^{(q)}_t / R) V[t]
// Two workgroups per CU: the 64 accumulator registers of O^T and the 32 of the Q operands leave no room for a
// third wavefront per SIMD (at 168 registers the compiler spills inside the tile loop).
#ifndef KVS_PQ_OUT_OCC
#define KVS_PQ_OUT_OCC 2
#endif
template <int D, bool COUNTS>
__global__ __launch_bounds__(kThreads, KVS_PQ_OUT_OCC) void pq_out_kernel(
    const UnitTable tab, const Shape sh, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, const int32_t* __restrict__ counts_in, const float* __restrict__ c_row,
    float* __restrict__ o_part, float* __restrict__ p_part) {
  typedef Tile<D> TL;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;                // 32-wide blocks of the value dimension
  __shared__ __attribute__((aligned(16))) unsigned char sm_k[2][TL::BYTES];
  __shared__ __attribute__((aligned(16))) unsigned char sm_v[2][TL::BYTES];
  __shared__ __attribute__((aligned(16))) float sm_lc[2][kTile], sm_ic[2][kTile];   // COUNTS: log2 c and 1 / c of the tile's rows
  __shared__ __attribute__((aligned(16))) float sm_cc[2][kTile];                    // COUNTS: c itself
  __shared__ uint4 sm_vt[2][DB][2][kWave];   // the V tile's blocks turned token-major: two operands per lane and block

  const int ui = find_unit(tab, blockIdx.x);
  const Unit un = tab.unit(ui);
  const int chunk = blockIdx.x - un.chunk_base;
  const int t0 = chunk * un.chunk_len;
  const int t1 = min(un.len, t0 + un.chunk_len);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int col = lane % 32, half = lane / 32;
  const int R = sh.R;
  const float sl2 = sh.scale_log2;
  const unsigned char* Kg = reinterpret_cast<const unsigned char*>(K + (size_t)un.in_row * D);
  const unsigned char* Vg = reinterpret_cast<const unsigned char*>(V + (size_t)un.in_row * D);
  const uint16_t* Qu = Q + (size_t)un.index * R * D;
  const int32_t* cnt = COUNTS ? counts_in + un.in_row : nullptr;

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

  // a tile always holds 32 whole rows: the ragged last one is moved back to end at the chunk's end and the
  // rows it shares with the tile before are skipped (every unit on this path has at least 32 rows)
  auto tile_base = [&](int j) { return min(t0 + j * kTile, t1 - kTile); };

  for (int qp = 0; qp < R; qp += kPassRows) {
    const int qrow = qp + 32 * wave + col;
    const bool ok = qrow < R;
    bf16x8 bq[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) bq[kk] = row_operand<D>(Qu, qrow, ok, kk, half);
    const float cq = ok ? c_row[(size_t)un.index * R + qrow] : INFINITY;   // exp2(-inf) = 0: no such row
    const int lim = last_seen_row(sh.causal, un.len, qrow);               // causal window: last row attended to
    f32x16 accO[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) accO[db] = zero;
    float wsum = 0.f;                       // sum of alpha / R over this lane's token rows, as the pairs hi + lo carry it

    typename TL::Regs rk = TL::load(Kg + (size_t)tile_base(0) * TL::ROWB, tid);
    typename TL::Regs rv = TL::load(Vg + (size_t)tile_base(0) * TL::ROWB, tid);
    for (int j = 0; j < ntiles; ++j) {
      const int buf = j & 1;
      TL::store(sm_k[buf], rk, tid);
      TL::store(sm_v[buf], rv, tid);
      if (COUNTS && tid < kTile) {
        const float c = (float)cnt[tile_base(j) + tid];
        sm_lc[buf][tid] = __builtin_amdgcn_logf(c);          // (base 2)
        sm_ic[buf][tid] = __builtin_amdgcn_rcpf(c);
        sm_cc[buf][tid] = c;
      }
      __syncthreads();
      const int shift = t0 + j * kTile - tile_base(j);       // leading rows that belong to the tile before
      {                                     // the next tile flies during this one (the last one is fetched twice)
        const int jn = min(j + 1, ntiles - 1);
        rk = TL::load(Kg + (size_t)tile_base(jn) * TL::ROWB, tid);
        rv = TL::load(Vg + (size_t)tile_base(jn) * TL::ROWB, tid);
        asm volatile("" ::: "memory");        // issue them here: sunk below the products they would be waited for at once
      }
      // The block V[tile rows, 32 w .. 32 w + 31] into the token-major operand layout, by wavefront w for all four
      // (every wavefront turning all blocks itself costs six more MFMAs and 48 conversions per tile and wavefront):
      // one product against the identity (exact: the values are bf16 numbers) leaves it in the accumulator layout,
      // which is the k-major operand layout of the product with P below.
      if (wave < DB) {
        f32x16 y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::operand(sm_v[buf], col, 2 * wave, half), ident[0], zero, 0, 0, 0);
        y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::operand(sm_v[buf], col, 2 * wave + 1, half), ident[1], y, 0, 0, 0);
        float yf[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) yf[v] = y[v];
        sm_vt[buf][wave][0][lane] = __builtin_bit_cast(uint4, pack8(yf));
        sm_vt[buf][wave][1][lane] = __builtin_bit_cast(uint4, pack8(yf + 8));
      }
      // logits of the tile against this wavefront's 32 query rows
      f32x16 acc = zero;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::operand(sm_k[buf], col, kk, half), bq[kk], acc, 0, 0, 0);
      // accumulator element v: token row 8 (v / 4) + 4 half + v % 4, query column `col`
      float p[16];
      if (COUNTS) {
        // (alpha / R) / c: the weight of the Value SUM of the row
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 lc = *reinterpret_cast<const float4*>(&sm_lc[buf][8 * g + 4 * half]);
          const float4 ic = *reinterpret_cast<const float4*>(&sm_ic[buf][8 * g + 4 * half]);
          p[4 * g] = ex2(fmaf(acc[4 * g], sl2, lc.x - cq)) * ic.x;
          p[4 * g + 1] = ex2(fmaf(acc[4 * g + 1], sl2, lc.y - cq)) * ic.y;
          p[4 * g + 2] = ex2(fmaf(acc[4 * g + 2], sl2, lc.z - cq)) * ic.z;
          p[4 * g + 3] = ex2(fmaf(acc[4 * g + 3], sl2, lc.w - cq)) * ic.w;
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) p[v] = ex2(fmaf(acc[v], sl2, -cq));
      }
      // rows of the tile before (a moved-back last tile) and rows behind the causal window's limit drop out;
      // both are rare and uniform per tile, so the common tile carries no per-element test
      if (shift > 0 || (sh.causal > 0 && tile_base(j) + kTile > un.len - sh.causal + 1)) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = 8 * (v / 4) + 4 * half + (v % 4);
          p[v] = (row >= shift && tile_base(j) + row <= lim) ? p[v] : 0.f;
        }
      }
      // as the operand of the next product, element i of k-step s is accumulator element 8 s + i
      bf16x8 ph[2], pl[2];
      float pw[16];
      split8w(p, ph[0], pl[0], pw);
      split8w(p + 8, ph[1], pl[1], pw + 8);
      if (COUNTS) {                         // (the pair carries (alpha / R) / c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 cc = *reinterpret_cast<const float4*>(&sm_cc[buf][8 * g + 4 * half]);
          wsum = fmaf(pw[4 * g], cc.x, wsum);
          wsum = fmaf(pw[4 * g + 1], cc.y, wsum);
          wsum = fmaf(pw[4 * g + 2], cc.z, wsum);
          wsum = fmaf(pw[4 * g + 3], cc.w, wsum);
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) wsum += pw[v];
      }
      __syncthreads();                      // the turned blocks are in place
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 vt0 = as_bf16x8(sm_vt[buf][db][0][lane]), vt1 = as_bf16x8(sm_vt[buf][db][1][lane]);
        accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt0, ph[0], accO[db], 0, 0, 0);
        accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt1, ph[1], accO[db], 0, 0, 0);
        accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt0, pl[0], accO[db], 0, 0, 0);
        accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt1, pl[1], accO[db], 0, 0, 0);
      }
    }
    __syncthreads();                        // the next pass starts with buffer 0 again
    wsum += __shfl_xor(wsum, 32, kWave);    // the other half's token rows
    if (ok && half == 0) p_part[(size_t)(un.chunk_base + chunk) * R + qrow] = wsum;
    if (ok) {
      float* dst = o_part + ((size_t)(un.chunk_base + chunk) * R + qrow) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 o4 = make_float4(accO[db][4 * g], accO[db][4 * g + 1], accO[db][4 * g + 2], accO[db][4 * g + 3]);
          *reinterpret_cast<float4*>(dst + 32 * db + 8 * g + 4 * half) = o4;
        }
      }
    }
  }
}

// o^{(q)} from the chunk partials and the sums of their weights (both in chunk order), as a bf16 pair hi + lo, and
// its squared norm.  One workgroup of D threads per (unit, query row).
template <int D>
__global__ __launch_bounds__(D) void pq_out_reduce_kernel(const UnitTable tab, const Shape sh,
                                                          const float* __restrict__ o_part,
                                                          const float* __restrict__ p_part,
                                                          uint16_t* __restrict__ o_hi, uint16_t* __restrict__ o_lo,
                                                          float* __restrict__ oo) {
  __shared__ float sm_ss[D / kWave];
  const int R = sh.R;
  const Unit un = tab.unit(blockIdx.x / R);
  const int q = blockIdx.x % R;
  const int d = threadIdx.x;
  float s = 0.f, w = 0.f;
#pragma unroll 8                            // (the loads of eight chunks in flight; the sums stay in chunk order)
  for (int c = 0; c < un.n_chunks; ++c) {
    s += o_part[((size_t)(un.chunk_base + c) * R + q) * D + d];
    w += p_part[(size_t)(un.chunk_base + c) * R + q];
  }
  const float m2o = -2.f * (s / w);                        // stored with the factor of ||v - o||^2 = ||v||^2 - 2 v.o + ||o||^2
  const uint32_t hi = f32_to_bf16(m2o);
  const uint32_t lo = f32_to_bf16(m2o - bf16_lo(hi));
  const size_t idx = ((size_t)un.index * R + q) * D + d;
  o_hi[idx] = (uint16_t)hi;
  o_lo[idx] = (uint16_t)lo;
  const float oe = -0.5f * (bf16_lo(hi) + bf16_lo(lo));    // the o the products below see
  float ss = oe * oe;
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) ss += __shfl_xor(ss, m, kWave);
  if (d % kWave == 0) sm_ss[d / kWave] = ss;
  __syncthreads();
  if (d == 0) {
    float t = sm_ss[0];
#pragma unroll
    for (int w = 1; w < D / kWave; ++w) t += sm_ss[w];
    oo[(size_t)un.index * R + q] = t;
  }
}

// ------------------------------------------------------------------------------------------------
// A_t and C_t of every token of the chunk.
//
// Both products are taken with the query rows as the accumulator ROWS: S'[q, t] = Q K^T, X'[q, t] = (-2 O) V^T.
// A lane then holds ONE token (column t = lane % 32) and 16 query rows, so the sums over q are plain
// register additions (plus one exchange between the wavefront's halves), and token t + 1 is the next lane
// (one DPP wavefront shift).  Per (t, q): one exp2, two square roots, eleven other instructions.
template <int D, bool COUNTS>
__global__ __launch_bounds__(kThreads, 2) void pq_norms_kernel(
    const UnitTable tab, const Shape sh, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, const int32_t* __restrict__ counts_in, const float* __restrict__ c_row,
    const uint16_t* __restrict__ o_hi,
    const uint16_t* __restrict__ o_lo, const float* __restrict__ oo, float* __restrict__ a_tok,
    float* __restrict__ c_edge) {
  typedef Tile<D> TL;
  constexpr int KS = D / 16;
  constexpr int STRIDE = kTile - 1;         // output rows per tile: the last row only serves as "next token"
  constexpr int PPT = TL::LPR / 8;          // pieces per thread when 8 threads share a row
  __shared__ __attribute__((aligned(16))) unsigned char sm_k[2][TL::BYTES];
  __shared__ __attribute__((aligned(16))) unsigned char sm_v[2][TL::BYTES];
  __shared__ float sm_vv[2][kTile + 1];                              // ||v_r||^2 (one spare entry: the last row's "next")
  __shared__ float sm_vd[2][kTile];                                  // v_r . v_{r+1}
  __shared__ float2 sm_out[2][kWaves][kTile];                        // (sum_q A, sum_q C) of every wavefront
  __shared__ __attribute__((aligned(16))) float sm_negc[kPassRows];  // per query row of the pass: -c[q]
  __shared__ __attribute__((aligned(16))) int sm_lim[kPassRows];     // causal window: last row attended to
  __shared__ float sm_lc[2][kTile + 1], sm_ic[2][kTile + 1];         // COUNTS: log2 c and 1 / c of the tile's rows

  const int ui = find_unit(tab, blockIdx.x);
  const Unit un = tab.unit(ui);
  const int chunk = blockIdx.x - un.chunk_base;
  const int t0 = chunk * un.chunk_len;
  const int t1 = min(un.len, t0 + un.chunk_len);
  const int ntiles = (t1 - t0 + STRIDE - 1) / STRIDE;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int col = lane % 32, half = lane / 32;
  const int R = sh.R;
  const float Rf = (float)R;
  const float sl2 = sh.scale_log2;
  const unsigned char* Kg = reinterpret_cast<const unsigned char*>(K + (size_t)un.in_row * D);
  const unsigned char* Vg = reinterpret_cast<const unsigned char*>(V + (size_t)un.in_row * D);
  const uint16_t* Qu = Q + (size_t)un.index * R * D;
  const uint16_t* Oh = o_hi + (size_t)un.index * R * D;
  const uint16_t* Ol = o_lo + (size_t)un.index * R * D;
  float* At = a_tok + un.in_row;
  float* Ce = c_edge + un.in_row;
  const int32_t* cnt = COUNTS ? counts_in + un.in_row : nullptr;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // Tile j puts out tokens t0 + 31 j .. + 30 and reads one row more.  Near the unit's end it is moved back
  // to hold 32 existing rows; the `shift` leading rows then belong to earlier tiles.
  auto tile_first = [&](int j) { return t0 + j * STRIDE; };
  auto tile_base = [&](int j) { return min(tile_first(j), un.len - kTile); };

  for (int qp = 0; qp < R; qp += kPassRows) {
    const int qrow = qp + 32 * wave + col;
    const bool ok = qrow < R;
    bf16x8 bq[KS], boh[KS], bol[KS];        // this wavefront's 32 query rows: Q, and -2 o as hi + lo
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      bq[kk] = row_operand<D>(Qu, qrow, ok, kk, half);
      boh[kk] = row_operand<D>(Oh, qrow, ok, kk, half);
      bol[kk] = row_operand<D>(Ol, qrow, ok, kk, half);
    }
    if (tid < kPassRows) {                  // (read after the first tile's barriers)
      const int q = qp + tid;
      sm_negc[tid] = (q < R) ? -c_row[(size_t)un.index * R + q] : -INFINITY;   // exp2(-inf) = 0: no such row
      sm_lim[tid] = last_seen_row(sh.causal, un.len, q);
    }
    // ||o^{(q)}||^2 of this lane's 16 accumulator rows: the value the X' accumulator starts from
    f32x16 oo_init;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int q = qp + 32 * wave + 8 * (v / 4) + 4 * half + (v % 4);
      oo_init[v] = (q < R) ? oo[(size_t)un.index * R + q] : 0.f;
    }

    // sums of the tile before -> memory (threads 0..31, one row each; the wavefronts in a fixed order)
    auto flush = [&](int j) {
      if (tid < kTile) {
        const int buf = j & 1;
        const int base = tile_base(j), shift = tile_first(j) - base;
        const int r = tid, t = base + r;
        if (r >= shift && r <= shift + STRIDE - 1 && t < t1) {
          float a = 0.f, c = 0.f;
          uint32_t mark = 0;                               // sign bit: some wavefront, or an earlier pass, marked the token
#pragma unroll
          for (int w = 0; w < kWaves; ++w) {
            const float2 o = sm_out[buf][w][r];
            mark |= __float_as_uint(o.x);
            a += fabsf(o.x);
            c += o.y;
          }
          if (r == kTile - 1) c = 0.f;                     // only the unit's last token: it has no next one
          if (qp > 0) {                                    // later passes add their query rows
            const float before = At[t];
            mark |= __float_as_uint(before);
            a += fabsf(before);
            c += Ce[t];
          }
          At[t] = __uint_as_float(__float_as_uint(a) | (mark & 0x80000000u));
          Ce[t] = c;
        }
      }
    };

    typename TL::Regs rk = TL::load(Kg + (size_t)tile_base(0) * TL::ROWB, tid);
    typename TL::Regs rv = TL::load(Vg + (size_t)tile_base(0) * TL::ROWB, tid);
    for (int j = 0; j < ntiles; ++j) {
      const int buf = j & 1;
      TL::store(sm_k[buf], rk, tid);
      TL::store(sm_v[buf], rv, tid);
      if (COUNTS && tid <= kTile) {           // (the spare entry stands for the last row's "next", which is never used)
        const float c = tid < kTile ? (float)cnt[tile_base(j) + tid] : 1.f;
        sm_lc[buf][tid] = __builtin_amdgcn_logf(c);          // (base 2)
        sm_ic[buf][tid] = __builtin_amdgcn_rcpf(c);
      }
      __syncthreads();
      {                                     // the next tile flies during this one (the last one is fetched twice)
        const int jn = min(j + 1, ntiles - 1);
        rk = TL::load(Kg + (size_t)tile_base(jn) * TL::ROWB, tid);
        rv = TL::load(Vg + (size_t)tile_base(jn) * TL::ROWB, tid);
        asm volatile("" ::: "memory");        // issue them here: sunk below the products they would be waited for at once
      }
      if (j > 0) flush(j - 1);
      // squared norms of the rows and of the sums of adjacent rows: eight threads per row
      {
        const int r = tid / 8, part = tid % 8;
        const int rn = min(r + 1, kTile - 1);
        float s_rr = 0.f, s_rn = 0.f;
#pragma unroll
        for (int x = 0; x < PPT; ++x) {           // (two bf16 products per instruction, added in fp32)
          const uint4 a = TL::piece_at(sm_v[buf], r, part * PPT + x);
          const uint4 b = TL::piece_at(sm_v[buf], rn, part * PPT + x);
          s_rr = dot2(a.x, a.x, s_rr); s_rn = dot2(a.x, b.x, s_rn);
          s_rr = dot2(a.y, a.y, s_rr); s_rn = dot2(a.y, b.y, s_rn);
          s_rr = dot2(a.z, a.z, s_rr); s_rn = dot2(a.z, b.z, s_rn);
          s_rr = dot2(a.w, a.w, s_rr); s_rn = dot2(a.w, b.w, s_rn);
        }
        s_rr = row_group_sum<8>(s_rr);
        s_rn = row_group_sum<8>(s_rn);
        if (part == 0) {
          sm_vv[buf][r] = s_rr;
          sm_vd[buf][r] = s_rn;
          if (r == kTile - 1) sm_vv[buf][kTile] = 0.f;       // read by the last column, whose edge is never used
        }
      }
      // S' = Q K^T and X' = (-2 O) V^T for this wavefront's 32 query rows
      f32x16 accS = zero, accX = COUNTS ? zero : oo_init;     // X'' = ||o||^2 - 2 v.o (COUNTS: -2 V.o, scaled below)
#pragma unroll
      for (int kk = 0; kk < KS; ++kk)
        accS = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[kk], TL::operand(sm_k[buf], col, kk, half), accS, 0, 0, 0);
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        const bf16x8 bv = TL::operand(sm_v[buf], col, kk, half);
        accX = __builtin_amdgcn_mfma_f32_32x32x16_bf16(boh[kk], bv, accX, 0, 0, 0);
        accX = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bol[kk], bv, accX, 0, 0, 0);
      }
      __syncthreads();                      // sm_vv / sm_vp of this tile are complete
      // accumulator element v: query row 32 wave + 8 (v / 4) + 4 half + v % 4 of the pass, token column `col`
      float vv = sm_vv[buf][col];
      float vp = fmaf(2.f, sm_vd[buf][col], vv + sm_vv[buf][col + 1]);         // ||v_t + v_{t+1}||^2
      float lc = 0.f, ic = 1.f;               // COUNTS: this lane's token stands for c tokens, v = V / c
      if (COUNTS) {
        lc = sm_lc[buf][col];
        ic = sm_ic[buf][col];
        const float icn = sm_ic[buf][col + 1];
        const float vvn = sm_vv[buf][col + 1] * icn * icn;
        vv = vv * ic * ic;
        vp = fmaf(2.f * ic * icn, sm_vd[buf][col], vv + vvn);
      }
      const int t_abs = tile_base(j) + col;
      float sumA = 0.f, sumC = 0.f;
      float leastA = INFINITY, leastC = INFINITY;   // smallest squared norms this lane forms in the tile (see below)
      // TAIL: the tile reaches into the causal window's masked rows (a uniform condition)
      auto rows = [&](auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int q0 = 32 * wave + 8 * g + 4 * half;
          const float4 nc4 = *reinterpret_cast<const float4*>(&sm_negc[q0]);
          const float nc[4] = {nc4.x, nc4.y, nc4.z, nc4.w};
          int lim[4] = {0, 0, 0, 0};
          if (TAIL) {
            const int4 l4 = *reinterpret_cast<const int4*>(&sm_lim[q0]);
            lim[0] = l4.x; lim[1] = l4.y; lim[2] = l4.z; lim[3] = l4.w;
          }
          float d2s[4], p2s[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int v = 4 * g + i;
            float a = ex2(fmaf(accS[v], sl2, COUNTS ? nc[i] + lc : nc[i]));  // alpha / R
            if (TAIL && t_abs > lim[i]) a = 0.f;
            const float x = COUNTS ? fmaf(accX[v], ic, oo_init[v]) : accX[v]; // ||o||^2 - 2 v_t . o
            // the same quantities of token t + 1: the next lane (the last column's are not used)
            const float a_n = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0x130, 0xF, 0xF, true));
            const float x_n = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x130, 0xF, 0xF, true));
            const float d2 = vv + x;                                       // ||v_t - o||^2
            const float p2 = fmaf(2.f, x + x_n, vp);                       // ||v_t + v_{t+1} - 2o||^2
            // (a rounding-size negative value stands for zero: the square roots take the magnitude)
            sumA = fmaf(a * fabsf(fmaf(-2.f * Rf, a, 1.f)), __builtin_amdgcn_sqrtf(fabsf(d2)), sumA);
            sumC = fmaf(a * a_n, __builtin_amdgcn_sqrtf(fabsf(p2)), sumC);
            d2s[i] = d2;
            p2s[i] = p2;
          }
          leastA = min3(min3(leastA, d2s[0], d2s[1]), d2s[2], d2s[3]);
          leastC = min3(min3(leastC, p2s[0], p2s[1]), p2s[2], p2s[3]);
          __builtin_amdgcn_sched_barrier(0);  // four rows at a time: interleaving all sixteen runs out of registers
        }
      };
      if (sh.causal > 0 && tile_base(j) + kTile > un.len - sh.causal + 1) rows(std::true_type{});
      else rows(std::false_type{});
      // Cancellation.  Where o^{(q)} comes close to v_t (a query row that puts nearly all its weight on one token) the
      // expansion above loses what is left of ||v_t - o||^2 to the rounding of its terms of size ||v_t||^2.  A token
      // one of whose squared norms falls below kCancel of its leading term is marked (the sign bit of its A_t, which
      // is never negative) and formed again by pq_redo_kernel, from differences.  The test costs one three-way
      // minimum per (t, q).
      int redo = (leastA < kCancel * vv || leastC < kCancel * vp) ? 1 : 0;
      redo |= __shfl_xor(redo, 32, kWave);
      sumA += __shfl_xor(sumA, 32, kWave);    // the other half's 16 query rows
      sumC += __shfl_xor(sumC, 32, kWave);
      if (half == 0) sm_out[buf][wave][col] = make_float2(redo ? -sumA : sumA, sumC * Rf);   // (sumA >= 0; -0 counts)
    }
    __syncthreads();
    flush(ntiles - 1);
    __syncthreads();                        // the next pass reuses the buffers
  }
}

// ------------------------------------------------------------------------------------------------
// Tokens that pq_norms_kernel marked (sign bit of A_t): A_t and C_t over all query rows once more, every squared norm
// as a sum of squared differences: ||v_t - o||^2 from v_t and the stored pair -2 o = hi + lo, likewise
// ||v_t + v_{t+1} - 2 o||^2.  One workgroup per span of kRedoSpan tokens; the span's marked tokens are listed and
// taken in turn: D / 8 adjacent lanes share a query row, eight dimensions each (one round of coalesced loads per row), the
// rows' terms are added per lane group in row order and the groups in a fixed butterfly order.  Every marked token leaves
// with a non-negative A_t, so no mark outlives this kernel.
template <int D, bool COUNTS>
__global__ __launch_bounds__(kThreads) void pq_redo_kernel(
    const UnitTable tab, const Shape sh, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, const int32_t* __restrict__ counts_in, const float* __restrict__ c_row,
    const uint16_t* __restrict__ o_hi, const uint16_t* __restrict__ o_lo, float* __restrict__ a_tok,
    float* __restrict__ c_edge) {
  constexpr int LPR = D / 8;                // lanes per query row
  constexpr int RPP = kThreads / LPR;       // query rows per pass of the workgroup
  __shared__ int sm_list[kRedoSpan];
  __shared__ int sm_n;
  __shared__ float sm_row[4][D];            // k_t, k_{t+1}, v_t, v_{t+1} (the Values divided by their cardinalities)
  __shared__ float sm_sum[2][kWaves];
  static_assert(kRedoSpan / kThreads <= 32, "one bit per token and thread");

  const Unit un = tab.unit(blockIdx.x);
  const int t0 = blockIdx.y * kRedoSpan;
  const int t1 = min(un.len, t0 + kRedoSpan);
  if (t0 >= t1) return;                     // (the grid is sized for the launch's longest unit)
  const int tid = threadIdx.x, part = tid % LPR;
  float* At = a_tok + un.in_row;
  float* Ce = c_edge + un.in_row;
  // nearly always no token of the span is marked: one look at all of them (bit k: token t0 + tid + 256 k)
  uint32_t marks = 0;
#pragma unroll
  for (int k = 0; k < kRedoSpan / kThreads; ++k) {
    const int t = t0 + tid + k * kThreads;
    if (t < t1) marks |= (__float_as_uint(At[t]) >> 31) << k;
  }
  if (!__syncthreads_or((int)marks)) return;
  if (tid == 0) sm_n = 0;
  __syncthreads();
  for (int k = 0; k < kRedoSpan / kThreads; ++k) {           // (any order: tokens are independent)
    if ((marks >> k) & 1) sm_list[atomicAdd(&sm_n, 1)] = t0 + tid + k * kThreads;
  }
  __syncthreads();
  const int n_marked = sm_n;
  const int R = sh.R;
  const float Rf = (float)R;
  const uint16_t* Kg = K + (size_t)un.in_row * D;
  const uint16_t* Vg = V + (size_t)un.in_row * D;
  const uint16_t* Qu = Q + (size_t)un.index * R * D + 8 * part;
  const uint16_t* Oh = o_hi + (size_t)un.index * R * D + 8 * part;
  const uint16_t* Ol = o_lo + (size_t)un.index * R * D + 8 * part;
  const float* cr = c_row + (size_t)un.index * R;

  {
    for (int m = 0; m < n_marked; ++m) {
      const int t = sm_list[m];
      const bool has_next = t + 1 < un.len;
      float lc = 0.f, lcn = 0.f;
      {
        float ic = 1.f, icn = 1.f;
        if (COUNTS) {
          const float c = (float)counts_in[un.in_row + t];
          const float cn = has_next ? (float)counts_in[un.in_row + t + 1] : 1.f;
          lc = __builtin_amdgcn_logf(c);                     // (base 2)
          lcn = __builtin_amdgcn_logf(cn);
          ic = __builtin_amdgcn_rcpf(c);
          icn = __builtin_amdgcn_rcpf(cn);
        }
        if (tid < 4 * LPR) {                  // one 16-byte piece per thread
          const int which = tid / LPR, pc = tid % LPR;
          float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          if (!(which & 1) || has_next) {
            const uint16_t* src = (which < 2 ? Kg : Vg) + (size_t)(t + (which & 1)) * D + 8 * pc;
            Piece<uint16_t>::unpack(*reinterpret_cast<const uint4*>(src), x);
          }
          const float f = which < 2 ? 1.f : ((which & 1) ? icn : ic);
#pragma unroll
          for (int i = 0; i < 8; ++i) sm_row[which][8 * pc + i] = x[i] * f;
        }
      }
      __syncthreads();
      float kt[8], kn[8], vt[8], vn[8];     // this lane's eight dimensions of the four rows
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        kt[i] = sm_row[0][8 * part + i];
        kn[i] = sm_row[1][8 * part + i];
        vt[i] = sm_row[2][8 * part + i];
        vn[i] = sm_row[3][8 * part + i];
      }
      float sumA = 0.f, sumC = 0.f;
      // (four passes of rows per trip, so that their loads are in flight together: the kernel's time is the latency
      // of these rounds; rows beyond R are computed on row 0's data and dropped)
      for (int q00 = 0; q00 < R; q00 += 4 * RPP) {
        uint4 rq[4], rh[4], rl[4];
        float rc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int q = q00 + u * RPP + tid / LPR;
          const int qc = q < R ? q : 0;
          rq[u] = *reinterpret_cast<const uint4*>(Qu + (size_t)qc * D);
          rh[u] = *reinterpret_cast<const uint4*>(Oh + (size_t)qc * D);
          rl[u] = *reinterpret_cast<const uint4*>(Ol + (size_t)qc * D);
          rc[u] = cr[qc];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int q = q00 + u * RPP + tid / LPR;
          const bool ok = q < R;              // (uniform over the lanes of a row, not over the wavefront: no branch around the sums)
          const int qc = ok ? q : 0;
          float qv[8], h[8], l[8];
          Piece<uint16_t>::unpack(rq[u], qv);
          Piece<uint16_t>::unpack(rh[u], h);
          Piece<uint16_t>::unpack(rl[u], l);
          float e = 0.f, en = 0.f, sA = 0.f, sC = 0.f;
  #pragma unroll
          for (int i = 0; i < 8; ++i) {
            e = fmaf(qv[i], kt[i], e);
            en = fmaf(qv[i], kn[i], en);
            const float m2o = h[i] + l[i];                                 // -2 o
            const float da = fmaf(0.5f, m2o, vt[i]);                       // v_t - o
            const float dc = vt[i] + vn[i] + m2o;                          // v_t + v_{t+1} - 2 o
            sA = fmaf(da, da, sA);
            sC = fmaf(dc, dc, sC);
          }
          e = row_group_sum<LPR>(e);
          en = row_group_sum<LPR>(en);
          sA = row_group_sum<LPR>(sA);
          sC = row_group_sum<LPR>(sC);
          const int lim = last_seen_row(sh.causal, un.len, qc);
          float a = ex2(fmaf(e, sh.scale_log2, lc - rc[u]));               // alpha / R
          float a_n = ex2(fmaf(en, sh.scale_log2, lcn - rc[u]));
          if (!ok || (sh.causal > 0 && t > lim)) a = 0.f;
          if (!has_next || (sh.causal > 0 && t + 1 > lim)) a_n = 0.f;
          sumA = fmaf(a * fabsf(fmaf(-2.f * Rf, a, 1.f)), __builtin_amdgcn_sqrtf(sA), sumA);
          sumC = fmaf(a * a_n, __builtin_amdgcn_sqrtf(sC), sumC);
        }
      }
      if (part != 0) sumA = sumC = 0.f;     // (all lanes of a row hold the same sums: one of them counts)
#pragma unroll
      for (int m2 = 32; m2 >= 1; m2 >>= 1) {
        sumA += __shfl_xor(sumA, m2, kWave);
        sumC += __shfl_xor(sumC, m2, kWave);
      }
      if (tid % kWave == 0) {
        sm_sum[0][tid / kWave] = sumA;
        sm_sum[1][tid / kWave] = sumC;
      }
      __syncthreads();
      if (tid == 0) {
        float a = sm_sum[0][0], c = sm_sum[1][0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) { a += sm_sum[0][w]; c += sm_sum[1][w]; }
        At[t] = a;
        Ce[t] = has_next ? c * Rf : 0.f;
      }
      __syncthreads();                      // sm_row and sm_sum are reused by the next token
    }
  }
}

template <int D, bool COUNTS>
hipError_t launch_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                    const int32_t* counts_in, const float* c_row, float* o_part, uint16_t* o_hi, uint16_t* o_lo,
                    float* oo, float* a_tok, float* c_edge, hipStream_t stream) {
  const dim3 grid(tab.total_chunks), block(kThreads);
  float* p_part = o_part + (size_t)tab.total_chunks * sh.R * D;   // the weights' sums lie behind the launch's partials
  hipLaunchKernelGGL((pq_out_kernel<D, COUNTS>), grid, block, 0, stream, tab, sh, (const uint16_t*)Q,
                     (const uint16_t*)K, (const uint16_t*)V, counts_in, c_row, o_part, p_part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((pq_out_reduce_kernel<D>), dim3(tab.n_units * sh.R), dim3(D), 0, stream, tab, sh, o_part, p_part,
                     o_hi, o_lo, oo);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((pq_norms_kernel<D, COUNTS>), grid, block, 0, stream, tab, sh, (const uint16_t*)Q,
                     (const uint16_t*)K, (const uint16_t*)V, counts_in, c_row, o_hi, o_lo, oo, a_tok, c_edge);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  int longest = 1;
  for (int u = 0; u < tab.n_units; ++u) longest = longest > tab.unit(u).len ? longest : tab.unit(u).len;
  const dim3 spans(tab.n_units, (longest + kRedoSpan - 1) / kRedoSpan);
  hipLaunchKernelGGL((pq_redo_kernel<D, COUNTS>), spans, block, 0, stream, tab, sh, (const uint16_t*)Q,
                     (const uint16_t*)K, (const uint16_t*)V, counts_in, c_row, o_hi, o_lo, a_tok, c_edge);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_per_query_norms(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                                  const int32_t* counts_in, const float* c_row, float* o_part, uint16_t* o_hi,
                                  uint16_t* o_lo, float* oo, float* a_tok, float* c_edge, hipStream_t stream) {
#define KVS_PQ_ARGS tab, sh, Q, K, V, counts_in, c_row, o_part, o_hi, o_lo, oo, a_tok, c_edge, stream
  if (counts_in) return sh.D == 64 ? launch_t<64, true>(KVS_PQ_ARGS) : launch_t<128, true>(KVS_PQ_ARGS);
  return sh.D == 64 ? launch_t<64, false>(KVS_PQ_ARGS) : launch_t<128, false>(KVS_PQ_ARGS);
#undef KVS_PQ_ARGS
}

}  // namespace kvs
