// Score kernels, MFMA path: bf16 inputs, query windows of at least 16 rows.
//
// Same two sweeps as the vector-ALU path (Sec. 4.1, Eq. attn_def_vec: logits, softmax over all
// cached Keys, here averaged over the unit's query rows): sweep 0 leaves per-chunk softmax
// statistics, sweep 1 recomputes the logits, writes alpha_bar and the chunk's share of o_bar.
//
// The logit tile is computed transposed, S^T[token, query] = K_tile * Q^T, with
// v_mfma_f32_32x32x16_bf16: the A operand is a 32-token tile of K, the B operand a block of
// 32 query rows.  The Q block of a wavefront (32*NT rows, NT <= 4) stays in registers for the whole
// sweep; K streams from HBM in coalesced 16-byte loads (16 lanes per 256-byte row), is staged in a
// wavefront-private, padded LDS region and read back in the operand layout.  In the accumulator
// a lane holds ONE query column and 16 token rows, so the running softmax statistics are
// lane-private (NT pairs per lane) and need no cross-lane traffic inside the loop; the sum over
// queries of sweep 1 is a 16-value reduce-scatter over 32 lanes (16 shuffles per tile).
//
// A workgroup has four wavefronts: WQ of them split the query rows (32*NT each), 4 / WQ split the
// chunk's 32-token tiles.  More than 128 * WQ query rows are handled in passes.
#include "kvs_device.h"

namespace kvs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kTile = 32;                 // tokens per MFMA tile

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D, int NT, int WQ, int PHASE>
__global__ __launch_bounds__(kThreads) void score_mfma_kernel(
    const UnitTable tab, const Shape sh, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, float* __restrict__ alpha_bar, float2* __restrict__ stats_part,
    float* __restrict__ o_part) {
  constexpr int WT = kWaves / WQ;           // wavefronts that split the tiles
  constexpr int KS = D / 16;                // MFMA k-steps per tile
  constexpr int LPR = D / 8;                // lanes per row when staging (16 bytes each)
  constexpr int RPI = kWave / LPR;          // rows per staging load instruction
  constexpr int NLD = kTile / RPI;          // staging loads per tile
  constexpr int STRIDE = D * 2 + 16;        // padded LDS row, bytes
  constexpr int QROWS = 32 * NT;            // query rows per wavefront
  constexpr int PASS_ROWS = QROWS * WQ;

  __shared__ __attribute__((aligned(16))) unsigned char sm_k[kWaves][kTile * STRIDE];
  __shared__ float sm_c[KVS_MAX_Q_ROWS];
  __shared__ float2 sm_stats[kWaves][QROWS];
  __shared__ float sm_alpha[kWaves][kTile];
  __shared__ float sm_o[kWaves][D];

  const int ui = find_unit(tab, blockIdx.x);
  const Unit un = tab.u[ui];
  const int chunk = blockIdx.x - un.chunk_base;
  const int t0 = chunk * un.chunk_len;
  const int t1 = min(un.len, t0 + un.chunk_len);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int iters = (ntiles + WT - 1) / WT;         // same trip count for every wavefront
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int wq = wave % WQ, wt = wave / WQ;
  const int col = lane % 32, half = lane / 32;
  const int R = sh.R;
  const float sl2 = sh.scale_log2;
  const size_t part_base = (size_t)un.index * kMaxChunks;

  const uint4* Kg = reinterpret_cast<const uint4*>(K + (size_t)un.in_row * D);
  const uint4* Vg = reinterpret_cast<const uint4*>(V + (size_t)un.in_row * D);
  const uint16_t* Qu = Q + (size_t)un.index * R * D;
  unsigned char* my_k = sm_k[wave];
  const int st_row = lane / LPR, st_piece = lane % LPR;

  if (PHASE == 1) {
    for (int q = tid; q < R; q += kThreads) {
      float M = -INFINITY;
      for (int c = 0; c < un.n_chunks; ++c) M = fmaxf(M, stats_part[(part_base + c) * R + q].x);
      float Z = 0.f;
      for (int c = 0; c < un.n_chunks; ++c) {
        const float2 s = stats_part[(part_base + c) * R + q];
        Z += s.y * ex2(s.x - M);
      }
      sm_c[q] = M + log2f(Z * (float)R);
    }
    __syncthreads();
  }

  float o_acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o_acc[i] = 0.f;

  for (int qp = 0; qp < R; qp += PASS_ROWS) {
    const bool first_pass = (qp == 0);
    const bool last_pass = (qp + PASS_ROWS >= R);

    // this wavefront's block of query rows, kept in registers as MFMA B operands
    bf16x8 bq[NT][KS];
    float cq[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int qrow = qp + wq * QROWS + nt * 32 + col;
      const bool ok = qrow < R;
      cq[nt] = (PHASE == 1 && ok) ? sm_c[qrow] : INFINITY;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (ok) raw = *reinterpret_cast<const uint4*>(Qu + (size_t)qrow * D + kk * 16 + 8 * half);
        bq[nt][kk] = *reinterpret_cast<bf16x8*>(&raw);
      }
    }

    float m_run[NT], l_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) { m_run[nt] = -INFINITY; l_run[nt] = 0.f; }

    // stage the first tile
    uint4 kreg[NLD];
    {
      const int j = wt;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int t = min(t0 + j * kTile + st_row + i * RPI, t1 - 1);
        kreg[i] = Kg[(size_t)t * LPR + st_piece];
      }
    }

    for (int it = 0; it < iters; ++it) {
      const int j = it * WT + wt;                   // tile index inside the chunk
      const int tile_t0 = t0 + j * kTile;
      const int nvalid = min(kTile, t1 - tile_t0);  // <= 0: this wavefront has no tile in this round

      // registers -> LDS (operand staging), then request the next tile and this tile's V rows
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        *reinterpret_cast<uint4*>(my_k + (st_row + i * RPI) * STRIDE + st_piece * 16) = kreg[i];
      }
      __syncthreads();
      {
        const int jn = j + WT;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          const int t = max(t0, min(t0 + jn * kTile + st_row + i * RPI, t1 - 1));
          kreg[i] = Kg[(size_t)t * LPR + st_piece];
        }
      }
      uint4 vreg[NLD];
      if (PHASE == 1 && last_pass && wq == 0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          const int t = max(t0, min(tile_t0 + st_row + i * RPI, t1 - 1));
          vreg[i] = Vg[(size_t)t * LPR + st_piece];
        }
      }

      // S^T tile = K_tile (32 x D) * Q_block^T (D x 32*NT)
      f32x16 acc[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nt][v] = 0.f;
      }
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(my_k + col * STRIDE + (kk * 16 + 8 * half) * 2);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[nt][kk], acc[nt], 0, 0, 0);
        }
      }
      // accumulator element v of a lane: token row 8*(v/4) + 4*half + v%4, query column `col`
      if (nvalid < kTile) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = 8 * (v / 4) + 4 * half + (v % 4);
          if (row >= nvalid) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[nt][v] = -INFINITY;
          }
        }
      }

      if (PHASE == 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          float tm = acc[nt][0];
#pragma unroll
          for (int v = 1; v < 16; ++v) tm = fmaxf(tm, acc[nt][v]);
          const float m_new = fmaxf(m_run[nt], tm * sl2);
          const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
          float s = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) s += ex2(fmaf(acc[nt][v], sl2, -m_safe));
          l_run[nt] = l_run[nt] * ex2(m_run[nt] - m_safe) + s;
          m_run[nt] = m_new;
        }
      } else {
        float p[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float s = 0.f;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) s += ex2(fmaf(acc[nt][v], sl2, -cq[nt]));
          p[v] = s;
        }
        // sum over the 32 query columns of each half: reduce-scatter, lane bits 4..1 pick v
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const bool up = lane & 16;
          const float send = up ? p[i] : p[i + 8];
          const float keep = up ? p[i + 8] : p[i];
          p[i] = keep + __shfl_xor(send, 16, kWave);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool up = lane & 8;
          const float send = up ? p[i] : p[i + 4];
          const float keep = up ? p[i + 4] : p[i];
          p[i] = keep + __shfl_xor(send, 8, kWave);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const bool up = lane & 4;
          const float send = up ? p[i] : p[i + 2];
          const float keep = up ? p[i + 2] : p[i];
          p[i] = keep + __shfl_xor(send, 4, kWave);
        }
        {
          const bool up = lane & 2;
          const float send = up ? p[0] : p[1];
          const float keep = up ? p[1] : p[0];
          p[0] = keep + __shfl_xor(send, 2, kWave);
        }
        p[0] += __shfl_xor(p[0], 1, kWave);
        const int v = (lane >> 1) & 15;
        const int row = 8 * (v / 4) + 4 * half + (v % 4);
        if ((lane & 1) == 0) sm_alpha[wave][row] = p[0];
        __syncthreads();
        if (wq == 0) {
          // rows of this tile: sum over the WQ wavefronts that share it, then over earlier passes
          float a_tok = 0.f;
          if (lane < kTile) {
#pragma unroll
            for (int w = 0; w < WQ; ++w) a_tok += sm_alpha[wave + w][lane];
            if (lane < nvalid) {
              float* dst = alpha_bar + un.in_row + tile_t0 + lane;
              if (!first_pass) a_tok += *dst;
              *dst = a_tok;
            } else {
              a_tok = 0.f;
            }
          }
          if (last_pass) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
              const float a_row = __shfl(a_tok, st_row + i * RPI, kWave);
              float vf[8];
              Piece<uint16_t>::unpack(vreg[i], vf);
#pragma unroll
              for (int e = 0; e < 8; ++e) o_acc[e] = fmaf(a_row, vf[e], o_acc[e]);
            }
          }
        }
      }
      __syncthreads();   // the LDS staging region and sm_alpha are rewritten in the next round
    }

    if (PHASE == 0) {
      // the two halves of a wavefront hold the same query column for different token rows
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const float m_o = __shfl_xor(m_run[nt], 32, kWave);
        const float l_o = __shfl_xor(l_run[nt], 32, kWave);
        const float m_n = fmaxf(m_run[nt], m_o);
        const float m_s = (m_n == -INFINITY) ? 0.f : m_n;
        l_run[nt] = l_run[nt] * ex2(m_run[nt] - m_s) + l_o * ex2(m_o - m_s);
        m_run[nt] = m_n;
        if (half == 0) sm_stats[wave][nt * 32 + col] = make_float2(m_run[nt], l_run[nt]);
      }
      __syncthreads();
      for (int i = tid; i < PASS_ROWS; i += kThreads) {
        const int q_wq = i / QROWS, q_in = i % QROWS;
        const int qrow = qp + i;
        if (qrow < R) {
          float M = -INFINITY;
#pragma unroll
          for (int w = 0; w < WT; ++w) M = fmaxf(M, sm_stats[w * WQ + q_wq][q_in].x);
          float Z = 0.f;
#pragma unroll
          for (int w = 0; w < WT; ++w) {
            const float2 s = sm_stats[w * WQ + q_wq][q_in];
            if (s.y > 0.f) Z += s.y * ex2(s.x - M);
          }
          stats_part[(part_base + chunk) * R + qrow] = make_float2(M, Z);
        }
      }
      __syncthreads();
    }
  }

  if (PHASE == 1) {
    // chunk share of o_bar: lanes with the same 16-byte piece, then the wavefronts
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
      for (int e = 0; e < 8; ++e) o_acc[e] += __shfl_xor(o_acc[e], off, kWave);
    }
    if (st_row == 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) sm_o[wave][st_piece * 8 + e] = o_acc[e];
    }
    __syncthreads();
    for (int d = tid; d < D; d += kThreads) {
      float s = 0.f;
      for (int w = 0; w < kWaves; ++w) s += sm_o[w][d];
      o_part[(part_base + chunk) * D + d] = s;
    }
  }
}

template <int D, int NT, int WQ>
hipError_t launch_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                    float* alpha_bar, const Workspace& ws, hipStream_t stream) {
  dim3 grid(tab.total_chunks), block(kThreads);
  hipLaunchKernelGGL((score_mfma_kernel<D, NT, WQ, 0>), grid, block, 0, stream, tab, sh, (const uint16_t*)Q,
                     (const uint16_t*)K, (const uint16_t*)V, alpha_bar, ws.stats_part, ws.o_part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((score_mfma_kernel<D, NT, WQ, 1>), grid, block, 0, stream, tab, sh, (const uint16_t*)Q,
                     (const uint16_t*)K, (const uint16_t*)V, alpha_bar, ws.stats_part, ws.o_part);
  return hipGetLastError();
}

template <int D>
hipError_t launch_d(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                    float* alpha_bar, const Workspace& ws, hipStream_t stream) {
  const int R = sh.R;
  if (R <= 32) return launch_t<D, 1, 1>(tab, sh, Q, K, V, alpha_bar, ws, stream);
  if (R <= 64) return launch_t<D, 2, 1>(tab, sh, Q, K, V, alpha_bar, ws, stream);
  if (R <= 128) return launch_t<D, 4, 1>(tab, sh, Q, K, V, alpha_bar, ws, stream);
  if (R <= 256) return launch_t<D, 4, 2>(tab, sh, Q, K, V, alpha_bar, ws, stream);
  return launch_t<D, 4, 4>(tab, sh, Q, K, V, alpha_bar, ws, stream);
}

}  // namespace

bool score_mfma_supported(const Shape& sh, kvs_dtype dt) { return dt == KVS_BF16 && sh.R >= 16; }

hipError_t launch_score_mfma(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                             float* alpha_bar, const Workspace& ws, hipStream_t stream) {
  return sh.D == 64 ? launch_d<64>(tab, sh, Q, K, V, alpha_bar, ws, stream)
                    : launch_d<128>(tab, sh, Q, K, V, alpha_bar, ws, stream);
}

}  // namespace kvs
