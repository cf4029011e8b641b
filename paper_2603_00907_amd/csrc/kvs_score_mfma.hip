// Score kernels, MFMA path: query windows of at least four rows (bf16; fp32 at the end of the file).
//
// Two sweeps over K (Sec. 4.1, Eq. attn_def_vec: logits, softmax over all cached Keys, here
// averaged over the unit's query rows): sweep 0 leaves per-chunk softmax statistics (running
// maximum and sum of exponentials, base-2 domain), a small kernel reduces them to one normaliser
// per query row and unit, sweep 1 recomputes the logits, normalises them and writes alpha_bar.
// (o_bar needs a pass over V: a streaming pass of its own beside the edge selection, see kvs_select.hip, or,
// in large launches of the kernel for 65..128 query rows, carried along by sweep 1.)
//
// The logit tile is computed transposed, S^T[token, query] = K_tile * Q^T, with
// v_mfma_f32_32x32x16_bf16: the A operand is a 32-token tile of K, the B operand a block of
// 32 query rows.  K streams from HBM straight into LDS (global_load_lds_dwordx4: 16 lanes fetch
// one 256-byte row, every instruction four whole rows) into a wavefront-private 8 KB tile; the
// 16-byte pieces of a row are stored XOR-swizzled by the row number so that the operand reads
// (ds_read_b128, 32 rows at the same piece) spread over all banks.  Wavefronts never wait for
// each other inside a sweep unless they share query rows.  In the accumulator a lane holds ONE
// query column and 16 token rows, so the running softmax statistics are lane-private; the sum
// over queries of sweep 1 is a 16-value reduce-scatter over 32 lanes (16 shuffles per tile), except in
// the wide kernel, whose sweep 1 takes the products the other way round (Q K^T): a lane then holds one
// token and the sum over queries is a sum over registers.
//
// A workgroup's wavefronts split the chunk's tiles.  Three kernels:
//   score_mfma_kernel       up to 64 query rows per wavefront, all register-stationary, two tile
//                           buffers per wavefront.  Windows of at most 64 rows (WQ = 1); on request also
//                           windows above 128 rows, where WQ wavefronts split the rows of a pass, share
//                           tiles and combine alpha_bar through LDS with a workgroup barrier per tile.
//   score_mfma_wide_kernel  more than 64 rows, in blocks of 64: up to 128 rows with one block
//                           register-stationary and one re-read from an LDS copy of the Q block for every
//                           tile, up to 256 rows with every block read from LDS (eight wavefronts), more
//                           rows as one launch per 256.
//   score_mfma_f32_kernel   fp32 inputs, v_mfma_f32_32x32x2_f32, 128 rows per launch.
// Rows of an already merged cache (cardinalities c given) enter with log2(c) added to the logit.
#include <cstdlib>
#include <type_traits>

#include "kvs_mfma_tile.h"

namespace kvs {
namespace {

using namespace mfma;

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

template <int D, int NT, int WQ, int PHASE>
__global__ __launch_bounds__(kThreads, 2) void score_mfma_kernel(
    const UnitTable tab, const Shape sh, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const int32_t* __restrict__ counts_in, float* __restrict__ alpha_bar, float2* __restrict__ stats_part,
    const float* __restrict__ c_row) {
  constexpr int WT = kWaves / WQ;           // wavefronts that split the tiles
  constexpr int KS = D / 16;                // MFMA k-steps per tile
  constexpr int LPR = D / 8;                // 16-byte pieces (= lanes) per row
  constexpr int RPI = kWave / LPR;          // rows per load instruction
  constexpr int NLD = kTile / RPI;          // load instructions per tile
  constexpr int ROWB = D * 2;               // bytes per row
  constexpr int QROWS = 32 * NT;            // query rows per wavefront
  constexpr int PASS_ROWS = QROWS * WQ;

  __shared__ __attribute__((aligned(1024))) unsigned char sm_k[kWaves][2][kTile * ROWB];
  __shared__ float sm_c[KVS_MAX_Q_ROWS];
  __shared__ float2 sm_stats[kWaves][QROWS];
  __shared__ float sm_alpha[kWaves][kTile];

  const int ui = find_unit(tab, blockIdx.x);
  const Unit un = tab.unit(ui);
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
  const int32_t* cnt = counts_in ? counts_in + un.in_row : nullptr;
  const float sc = cnt ? 1.f : sl2;        // the accumulators hold finished logits when cardinalities were added
  const size_t part_base = (size_t)un.index * kMaxChunks;

  const uint4* Kg = reinterpret_cast<const uint4*>(K + (size_t)un.in_row * D);
  const uint16_t* Qu = Q + (size_t)un.index * R * D;
  unsigned char* my_k = sm_k[wave][0];        // two tile buffers per wavefront: my_k, my_k + TILEB
  constexpr int TILEB = kTile * ROWB;
  // staging: lane -> (row within the instruction's block of RPI rows, LDS slot); the piece fetched
  // into slot s of row r is s ^ (r % LPR)
  const int st_row = lane / LPR, st_slot = lane % LPR;

  // byte offset of this lane's piece inside a full tile, for each of the NLD load instructions
  int ld_off[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int row = st_row + i * RPI;
    ld_off[i] = row * ROWB + (st_slot ^ (row % LPR)) * 16;
  }
  // LDS byte addresses of this lane's A operands (k-step kk) in tile buffer 0
  uint32_t a_addr[KS];
  {
    const uint32_t base = (uint32_t)(size_t)KVS_LDS_PTR(my_k) + col * ROWB;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) a_addr[kk] = base + ((2 * kk + half) ^ (col % LPR)) * 16;
  }
  // A tile always holds 32 whole rows of the chunk: the ragged last tile is moved back so that it ends
  // at the chunk's end, and the rows it shares with the tile before it are masked out (`shift` of
  // them).  Every unit has at least 32 tokens on this path, so the moved tile stays inside the unit.
  auto issue_tile = [&](int j, int buf) {
    const int tile_t0 = t0 + j * kTile;
    if (tile_t0 >= t1) return false;          // no such tile
    const int base_t = min(tile_t0, t1 - kTile);
    const unsigned char* base = reinterpret_cast<const unsigned char*>(Kg) + (size_t)base_t * ROWB;
    // a launch larger than the caches streams K past them in sweep 0 (the cache-policy bit is an immediate: two
    // copies); sweep 1 leaves what it can of K in the memory-side cache for the merge pass
    if (sh.stream && PHASE == 0) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        __builtin_amdgcn_global_load_lds(KVS_GLOBAL_PTR(base + ld_off[i]),
                                         KVS_LDS_PTR(my_k + buf * TILEB + i * 1024), 16, 0, kNonTemporal);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        __builtin_amdgcn_global_load_lds(KVS_GLOBAL_PTR(base + ld_off[i]),
                                         KVS_LDS_PTR(my_k + buf * TILEB + i * 1024), 16, 0, 0);
      }
    }
    return true;
  };

  if (PHASE == 1) load_row_consts(c_row, un.index, R, sm_c);

  for (int qp = 0; qp < R; qp += PASS_ROWS) {
    const bool first_pass = (qp == 0);

    issue_tile(wt, 0);                        // flies while the Q block is fetched

    // this wavefront's block of query rows, kept in registers as MFMA B operands
    bf16x8 bq[NT][KS];
    float cq[NT];
    if (WQ == 1) {
      // One coalesced, swizzled copy of the block in LDS per workgroup, then operand reads from LDS:
      // 4x less L2 traffic than per-wavefront row gathers.  Every wavefront fetches a quarter of the
      // rows into its own second tile buffer, which is idle until the operands are in registers.
      constexpr int RW = QROWS / kWaves;              // rows staged per wavefront
      constexpr int QLD = RW / RPI > 0 ? RW / RPI : 1;
      const uint4* Qg = reinterpret_cast<const uint4*>(Qu);
#pragma unroll
      for (int i = 0; i < QLD; ++i) {
        const int lr = i * RPI + st_row;              // local row in this wavefront's buffer
        const int qrow = min(qp + wave * RW + min(lr, RW - 1), R - 1);   // rows past R repeat the last row
        const int piece = st_slot ^ (lr % LPR);
        __builtin_amdgcn_global_load_lds(KVS_GLOBAL_PTR(Qg + (size_t)qrow * LPR + piece),
                                         KVS_LDS_PTR(my_k + TILEB + i * 1024), 16, 0, 0);
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0)
      __syncthreads();
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int row = nt * 32 + col;
        const int lr = row % RW;
        const unsigned char* src = sm_k[row / RW][1] + lr * ROWB;
        cq[nt] = (PHASE == 1 && qp + row < R) ? sm_c[qp + row] : INFINITY;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
          const int slot = (2 * kk + half) ^ (lr % LPR);
          bq[nt][kk] = *reinterpret_cast<const bf16x8*>(src + slot * 16);
        }
      }
      __syncthreads();                                // the second buffers go back to the K tiles
    } else {
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
    }
    int lim[NT];                                      // causal window: last row each query column attends to
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) lim[nt] = last_seen_row(sh.causal, un.len, qp + wq * QROWS + nt * 32 + col);
    bool next_in_flight = (iters > 1) && issue_tile(wt + WT, 1);   // loads of the tile after the current one

    float m_run[NT], l_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) { m_run[nt] = -INFINITY; l_run[nt] = 0.f; }

    for (int it = 0; it < iters; ++it) {
      const int j = it * WT + wt;                   // tile index inside the chunk
      const int tile_t0 = t0 + j * kTile;
      const int base_t = min(tile_t0, t1 - kTile);  // first token of the (possibly moved back) tile
      const int shift = (tile_t0 >= t1) ? kTile : tile_t0 - base_t;   // leading rows that are not ours
      if (WQ == 1 && shift == kTile) break;         // this wavefront has run out of tiles

      // wait for this tile only (loads return in order: at most the NLD loads of the next tile may
      // still be in flight); first half of the k-steps: operands to registers, MFMAs
      if (next_in_flight) __builtin_amdgcn_s_waitcnt(0x0F70 | (NLD & 15) | ((NLD >> 4) << 14));   // vmcnt(NLD)
      else __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
      asm volatile("" ::: "memory");
      static_assert(KS == 4 || KS == 8, "operand reads come in groups of four");
      constexpr int KH = 4;
      f32x16 acc[NT];
      {
        bf16x8 a[KH];
        if (it & 1) lds_read_4x16<TILEB>(a[0], a[1], a[2], a[3], a_addr);
        else lds_read_4x16<0>(a[0], a[1], a[2], a[3], a_addr);
        if (KS == 4) next_in_flight = (it + 2 < iters) && issue_tile(j + 2 * WT, it & 1);
#pragma unroll
        for (int kk = 0; kk < KH; ++kk) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            if (kk == 0) {
              const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
              acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], bq[nt][kk], zero, 0, 0, 0);
            } else {
              acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], bq[nt][kk], acc[nt], 0, 0, 0);
            }
          }
        }
      }
      // second half; once its operands have left LDS the tile buffer goes to the load after next
      if (KS == 8) {
        bf16x8 a[KH];
        if (it & 1) lds_read_4x16<TILEB>(a[0], a[1], a[2], a[3], a_addr + (KS == 8 ? 4 : 0));
        else lds_read_4x16<0>(a[0], a[1], a[2], a[3], a_addr + (KS == 8 ? 4 : 0));
        next_in_flight = (it + 2 < iters) && issue_tile(j + 2 * WT, it & 1);
#pragma unroll
        for (int kk = 0; kk < KH; ++kk) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], bq[nt][(kk + KH) % KS], acc[nt], 0, 0, 0);
          }
        }
      }
      // accumulator element v of a lane: token row 8*(v/4) + 4*half + v%4, query column `col`
      if (shift > 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = 8 * (v / 4) + 4 * half + (v % 4);
          if (row < shift) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[nt][v] = -INFINITY;
          }
        }
      }
      if (sh.causal > 0 && base_t + kTile > un.len - sh.causal + 1) mask_causal<NT>(acc, lim, base_t, half);

      if (cnt) logits_with_counts<NT>(acc, cnt, base_t, half, sl2);
      if (PHASE == 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          float tm = acc[nt][0];
#pragma unroll
          for (int v = 1; v < 16; ++v) tm = fmaxf(tm, acc[nt][v]);
          const float m_new = fmaxf(m_run[nt], tm * sc);
          const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
          float s = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) s += ex2(fmaf(acc[nt][v], sc, -m_safe));
          l_run[nt] = l_run[nt] * ex2(m_run[nt] - m_safe) + s;
          m_run[nt] = m_new;
        }
      } else {
        float p[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float s = 0.f;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) s += ex2(fmaf(acc[nt][v], sc, -cq[nt]));
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
        float a_tok = p[0];
        if (WQ > 1) {
          // the WQ wavefronts that share this tile add their query blocks up through LDS
          if ((lane & 1) == 0) sm_alpha[wave][row] = a_tok;
          __syncthreads();
          if (wq == 0 && lane < kTile) {
            a_tok = 0.f;
#pragma unroll
            for (int w = 0; w < WQ; ++w) a_tok += sm_alpha[wave + w][lane];
            if (lane >= shift) {
              float* dst = alpha_bar + un.in_row + base_t + lane;
              if (!first_pass) a_tok += *dst;
              *dst = a_tok;
            }
          }
          __syncthreads();
        } else if ((lane & 1) == 0 && row >= shift) {
          float* dst = alpha_bar + un.in_row + base_t + row;
          if (!first_pass) a_tok += *dst;
          *dst = a_tok;
        }
      }
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
}

// 65..256 query rows in ONE pass over K, as QB blocks of 64 rows (QB = 2: up to 128 rows, four wavefronts per
// workgroup, two workgroups per CU; QB = 3, 4: up to 192 / 256 rows, eight wavefronts per workgroup and one workgroup
// per CU, because the Q block then takes 48 / 64 KB of LDS).  All rows' operands plus the accumulators do not fit the
// registers of a wavefront at two wavefronts per SIMD, so only rows 0..63 are register-stationary (QB = 2; none
// with more blocks); the others stay in the workgroup's swizzled LDS copy of the Q block and are re-read for every
// tile (16 KB of LDS reads per block and tile, hidden behind the MFMAs already in the pipe).  The K tile is
// moved to registers whole (all k-steps) at the start of a tile, which frees its single LDS buffer
// for the wavefront's next tile at once: that load flies during both halves' MFMAs and softmax work.
// OBAR (sweep 1 only): the pass over V that o_bar = sum_t alpha_bar[t] V[t] needs rides along.  A tile's Value
// rows are requested when the tile starts and used when its alpha_bar values exist, one tile of arithmetic
// later, so they cost no waiting, and they travel while the sweep's own loads are idle behind its arithmetic.
// Every workgroup leaves the sum over its chunk in o_part[unit][chunk]; consumers add the chunks in order.
// MULTI: more than 256 query rows, one launch per 256 of them (rows qp0 .. qp0 + 255 of every unit): sweep 0 leaves
// each launch's rows' statistics, sweep 1 adds its rows' share to what the launches before left in alpha_bar, and
// the last launch (which alone may carry the pass over V) applies the cardinalities.
template <int D, int PHASE, bool STREAM, bool CAUSAL, bool OBAR, int QB, bool MULTI = false>
__global__ __launch_bounds__(QB == 2 ? 256 : 512, QB == 2 ? 2 : 1) void score_mfma_wide_kernel(
    const UnitTable tab, const Shape sh, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const int32_t* __restrict__ counts_in, float* __restrict__ alpha_bar, float2* __restrict__ stats_part,
    const float* __restrict__ c_row, const uint16_t* __restrict__ V, float* __restrict__ o_part, const int qp0) {
  static_assert(!MULTI || QB == 4, "passes of 256 rows");
  const int qp = MULTI ? qp0 : 0;           // first query row of this launch
  static_assert(!OBAR || PHASE == 1, "the Value pass belongs to sweep 1");
  constexpr int KS = D / 16;
  constexpr int LPR = D / 8;
  constexpr int RPI = kWave / LPR;
  constexpr int NLD = kTile / RPI;
  constexpr int ROWB = D * 2;
  constexpr int TILEB = kTile * ROWB;
  constexpr int QROWS = 64 * QB;            // query rows per wavefront (QB blocks of 64)
  constexpr int NW = QB == 2 ? 4 : 8;       // wavefronts per workgroup
  constexpr int NTHR = NW * kWave;
  static_assert(QB >= 2 && QB <= 4, "the Q block must fit the LDS beside the tile buffers");
  static_assert(KS == 4 || KS == 8, "operand reads come in groups of four");

  __shared__ __attribute__((aligned(1024))) unsigned char sm_k[NW][TILEB];
  __shared__ __attribute__((aligned(1024))) unsigned char sm_q[QROWS * ROWB];
  __shared__ float2 sm_stats[NW][QROWS];
  __shared__ __attribute__((aligned(16))) float sm_cq[QROWS];     // sweep 1: the rows' normalisers ...
  __shared__ __attribute__((aligned(16))) int sm_lim[QROWS];      // ... and the last row each attends to

  const int ui = find_unit(tab, blockIdx.x);
  const Unit un = tab.unit(ui);
  const int chunk = blockIdx.x - un.chunk_base;
  const int t0 = chunk * un.chunk_len;
  const int t1 = min(un.len, t0 + un.chunk_len);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int iters = (ntiles + NW - 1) / NW;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int col = lane % 32, half = lane / 32;
  const int R = sh.R;
  const float sl2 = sh.scale_log2;
  const int32_t* cnt = counts_in ? counts_in + un.in_row : nullptr;
  const float sc = cnt ? 1.f : sl2;        // the accumulators hold finished logits when cardinalities were added
  const size_t part_base = (size_t)un.index * kMaxChunks;

  const unsigned char* Kg = reinterpret_cast<const unsigned char*>(K + (size_t)un.in_row * D);
  const uint4* Qg = reinterpret_cast<const uint4*>(Q + (size_t)un.index * R * D);
  unsigned char* my_k = sm_k[wave];
  const int st_row = lane / LPR, st_slot = lane % LPR;

  int ld_off[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int row = st_row + i * RPI;
    ld_off[i] = row * ROWB + (st_slot ^ (row % LPR)) * 16;
  }
  // LDS byte addresses of this lane's operand pieces: K tile row `col`, Q block row `col` (+ 32, 64, 96)
  uint32_t a_addr[KS], q_addr[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    const uint32_t off = col * ROWB + ((2 * kk + half) ^ (col % LPR)) * 16;
    a_addr[kk] = (uint32_t)(size_t)KVS_LDS_PTR(my_k) + off;
    q_addr[kk] = (uint32_t)(size_t)KVS_LDS_PTR(sm_q) + off;
  }
  // the ragged last tile is moved back to end at the chunk's end, see score_mfma_kernel
  auto issue_tile = [&](int j) {
    const int tile_t0 = t0 + j * kTile;
    if (tile_t0 >= t1) return false;
    const int base_t = min(tile_t0, t1 - kTile);
    const unsigned char* base = Kg + (size_t)base_t * ROWB;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      // (sweep 1 keeps the ordinary policy: what it leaves of K in the memory-side cache is what the merge
      // pass, two short launches later, starts from: 3 % of the step on one stream, 1 % on two)
      __builtin_amdgcn_global_load_lds(KVS_GLOBAL_PTR(base + ld_off[i]), KVS_LDS_PTR(my_k + i * 1024), 16, 0,
                                       (STREAM && PHASE == 0) ? kNonTemporal : 0);
    }
    return true;
  };

  // Sweep 1 takes the products the other way round (query rows as accumulator rows, see below), so the
  // normalisers (written by the finalize kernel between the sweeps) are indexed by accumulator element and come
  // from LDS.  exp2(-inf) = 0: a row that does not exist adds nothing.
  if (PHASE == 1) {
    if (tid < QROWS) {
      sm_cq[tid] = (qp + tid < R) ? c_row[(size_t)un.index * R + qp + tid] : INFINITY;
      sm_lim[tid] = last_seen_row(CAUSAL ? sh.causal : 0, un.len, qp + tid);
    }
    __syncthreads();
  }

  int lim[2 * QB];                          // causal window: last row each of the lane's query columns attends to
#pragma unroll
  for (int b = 0; b < 2 * QB; ++b) lim[b] = last_seen_row(CAUSAL ? sh.causal : 0, un.len, qp + b * 32 + col);

  // the Q block, once per workgroup: every wavefront fetches its share of the rows (rows past R repeat the last one)
  {
    constexpr int RPW = QROWS / NW;           // 32 or 24 rows
    constexpr int QLD = RPW / RPI;
    static_assert(RPW % RPI == 0, "whole load instructions");
#pragma unroll
    for (int i = 0; i < QLD; ++i) {
      const int lr = wave * RPW + i * RPI + st_row;
      const int qrow = min(qp + lr, R - 1);
      const int piece = st_slot ^ (lr % LPR);
      __builtin_amdgcn_global_load_lds(KVS_GLOBAL_PTR(Qg + (size_t)qrow * LPR + piece),
                                       KVS_LDS_PTR(sm_q + (wave * RPW + i * RPI) * ROWB), 16, 0, 0);
    }
  }
  // first K tile flies while Q lands; loads return in order, so leaving NLD in flight means Q is there
  if (issue_tile(wave)) __builtin_amdgcn_s_waitcnt(0x0F70 | (NLD & 15) | ((NLD >> 4) << 14));
  else __builtin_amdgcn_s_waitcnt(0x0F70);
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  bf16x8 bq[2][KS];                         // rows 0..63, register-stationary (two blocks only: with more, the
                                            // statistics of eight column blocks take the registers and every block
                                            // is read from LDS)
#pragma unroll
  for (int g = 0; g < (QB == 2 ? KS / 4 : 0); ++g) {
    lds_read_4x16<0>(bq[0][4 * g], bq[0][4 * g + 1], bq[0][4 * g + 2], bq[0][4 * g + 3], q_addr + 4 * g);
    lds_read_4x16<32 * ROWB>(bq[1][4 * g], bq[1][4 * g + 1], bq[1][4 * g + 2], bq[1][4 * g + 3], q_addr + 4 * g);
  }

  float m_run[2 * QB], l_run[2 * QB];
#pragma unroll
  for (int b = 0; b < 2 * QB; ++b) { m_run[b] = -INFINITY; l_run[b] = 0.f; }
  // OBAR: this lane's 16-byte piece of sum_t w_t V[t] over the wavefront's tiles (w = alpha_bar, or alpha_bar / c)
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  float o_acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o_acc[e] = 0.f;
  const unsigned char* Vg = OBAR ? reinterpret_cast<const unsigned char*>(V + (size_t)un.in_row * D) : nullptr;

  for (int it = 0; it < iters; ++it) {
    const int j = it * NW + wave;
    const int tile_t0 = t0 + j * kTile;
    if (tile_t0 >= t1) break;                       // this wavefront has run out of tiles
    const int base_t = min(tile_t0, t1 - kTile);
    const int shift = tile_t0 - base_t;             // leading rows that belong to the tile before

    __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): this tile (nothing else is in flight)
    asm volatile("" ::: "memory");
    bf16x8 a[KS];
#pragma unroll
    for (int g = 0; g < KS / 4; ++g)
      lds_read_4x16<0>(a[4 * g], a[4 * g + 1], a[4 * g + 2], a[4 * g + 3], a_addr + 4 * g);
    issue_tile(j + NW);                         // the buffer is free again
    // OBAR: the tile's Value rows, RPI whole rows per load; they are used at the end of the tile
    u32x4 vr[NLD];
    if (OBAR) {
      const unsigned char* vt = Vg + (size_t)base_t * ROWB + lane * 16;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const u32x4* src = reinterpret_cast<const u32x4*>(vt + i * 1024);
        vr[i] = STREAM ? __builtin_nontemporal_load(src) : *src;
      }
    }

    float p_tok = 0.f;                              // sweep 1: this lane's token, summed over its query rows
    // one block of 64 query rows; the block number is a compile-time constant so that the operand reads of the
    // blocks kept in LDS address them with immediate offsets (no address registers per block)
    // NTB: column blocks of 32 rows that exist in this block of 64 (the last block may hold one only)
    auto block = [&](auto hc, auto ntc) {
      constexpr int h = decltype(hc)::value;
      constexpr int NTB = decltype(ntc)::value;
      f32x16 acc[2];
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if (h == 0 && QB == 2) {
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
#pragma unroll
          for (int nt = 0; nt < 2; ++nt) {
            acc[nt] = (PHASE == 0)
                ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], bq[nt][kk], kk == 0 ? zero : acc[nt], 0, 0, 0)
                : __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[nt][kk], a[kk], kk == 0 ? zero : acc[nt], 0, 0, 0);
          }
        }
      } else if (NTB == 1) {
        acc[1] = zero;
#pragma unroll
        for (int kp = 0; kp < KS / 2; ++kp) {
          bf16x8 b00, b10;
          lds_read_2x1<64 * h * ROWB>(b00, b10, q_addr[2 * kp], q_addr[2 * kp + 1]);
          if (PHASE == 0) {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 * kp], b00, kp == 0 ? zero : acc[0], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 * kp + 1], b10, acc[0], 0, 0, 0);
          } else {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b00, a[2 * kp], kp == 0 ? zero : acc[0], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b10, a[2 * kp + 1], acc[0], 0, 0, 0);
          }
        }
      } else {
#pragma unroll
        for (int kp = 0; kp < KS / 2; ++kp) {
          bf16x8 b00, b01, b10, b11;
          lds_read_2x2<64 * h * ROWB, (64 * h + 32) * ROWB>(b00, b01, b10, b11, q_addr[2 * kp], q_addr[2 * kp + 1]);
          if (PHASE == 0) {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 * kp], b00, kp == 0 ? zero : acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 * kp], b01, kp == 0 ? zero : acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 * kp + 1], b10, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 * kp + 1], b11, acc[1], 0, 0, 0);
          } else {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b00, a[2 * kp], kp == 0 ? zero : acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b01, a[2 * kp], kp == 0 ? zero : acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b10, a[2 * kp + 1], acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b11, a[2 * kp + 1], acc[1], 0, 0, 0);
          }
        }
      }
      if (PHASE == 0) {
        // accumulator element v of a lane: token row 8*(v/4) + 4*half + v%4, query column `col`
        if (shift > 0) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v / 4) + 4 * half + (v % 4);
            if (row < shift) { acc[0][v] = -INFINITY; acc[1][v] = -INFINITY; }
          }
        }
        if (CAUSAL && base_t + kTile > un.len - sh.causal + 1) {
          const int lim2[2] = {lim[2 * h], lim[2 * h + 1]};
          mask_causal<2>(acc, lim2, base_t, half);
        }
        if (cnt) logits_with_counts<2>(acc, cnt, base_t, half, sl2);
#pragma unroll
        for (int nt = 0; nt < NTB; ++nt) {
          const int b = 2 * h + nt;
          float tm = acc[nt][0];
#pragma unroll
          for (int v = 1; v < 16; ++v) tm = fmaxf(tm, acc[nt][v]);
          const float m_new = fmaxf(m_run[b], tm * sc);
          const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
          float s = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) s += ex2(fmaf(acc[nt][v], sc, -m_safe));
          l_run[b] = l_run[b] * ex2(m_run[b] - m_safe) + s;
          m_run[b] = m_new;
        }
      } else {
        // Sweep 1, products taken as Q K^T: accumulator element v of block nt is query row
        // 32 (2 h + nt) + 8 (v / 4) + 4 half + v % 4, and the lane's column is ONE token, so the sum over the
        // query rows is a sum over registers
        const bool tail = CAUSAL && base_t + kTile > un.len - sh.causal + 1;       // uniform
#pragma unroll
        for (int nt = 0; nt < NTB; ++nt) {
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int q0 = 32 * (2 * h + nt) + 8 * g + 4 * half;
            const float4 c4 = *reinterpret_cast<const float4*>(&sm_cq[q0]);
            const float cq[4] = {c4.x, c4.y, c4.z, c4.w};
            float e[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) e[i] = ex2(fmaf(acc[nt][4 * g + i], sl2, -cq[i]));
            if (tail) {
              const int4 l4 = *reinterpret_cast<const int4*>(&sm_lim[q0]);
              const int lq[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
              for (int i = 0; i < 4; ++i) e[i] = (base_t + col > lq[i]) ? 0.f : e[i];
            }
            p_tok += (e[0] + e[1]) + (e[2] + e[3]);
          }
        }
      }
    };
    typedef std::integral_constant<int, 1> one_t;
    typedef std::integral_constant<int, 2> two_t;
    block(std::integral_constant<int, 0>{}, two_t{});
    if constexpr (QB == 2) {
      block(std::integral_constant<int, 1>{}, two_t{});
    } else {
      // the last block holds one or two column blocks of 32 rows (uniform)
      block(std::integral_constant<int, 1>{}, two_t{});
      if constexpr (QB == 4) block(std::integral_constant<int, 2>{}, two_t{});
      if (R - qp > 64 * (QB - 1) + 32) block(std::integral_constant<int, QB - 1>{}, two_t{});
      else block(std::integral_constant<int, QB - 1>{}, one_t{});
    }

    if (PHASE == 1) {
      // the two halves of the wavefront hold the token's other query rows; a row that stands for c tokens has
      // c equal terms in every softmax sum (2^(e + log2 c) = c 2^e)
      p_tok += __shfl_xor(p_tok, 32, kWave);
      if (MULTI && qp > 0) p_tok += alpha_bar[un.in_row + base_t + col];     // the rows of the launches before
      if (OBAR) {
        // lane l holds the weight of tile row l % 32; load i of this lane is row i * RPI + st_row
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          const int row = i * RPI + st_row;
          float w = __shfl(p_tok, row, kWave);
          if (row < shift) w = 0.f;                         // the tile before has counted this row
          float vf[8];
          Piece<uint16_t>::unpack(make_uint4(vr[i].x, vr[i].y, vr[i].z, vr[i].w), vf);
#pragma unroll
          for (int e = 0; e < 8; ++e) o_acc[e] = fmaf(w, vf[e], o_acc[e]);
        }
      }
      if (cnt && (!MULTI || qp + QROWS >= R)) p_tok *= (float)cnt[base_t + col];
      if (half == 0 && col >= shift) alpha_bar[un.in_row + base_t + col] = p_tok;
    }
  }

  if (OBAR) {
    // lanes that hold the same piece of the row, then the wavefronts, in a fixed order
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
      for (int e = 0; e < 8; ++e) o_acc[e] += __shfl_xor(o_acc[e], off, kWave);
    }
    float* sm_o = reinterpret_cast<float*>(&sm_stats[0][0]);          // (sweep 0's table, idle in sweep 1)
    if (st_row == 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) sm_o[wave * D + st_slot * 8 + e] = o_acc[e];
    }
    __syncthreads();
    if (tid < D) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) sum += sm_o[w * D + tid];
      o_part[((size_t)un.index * kMaxChunks + chunk) * D + tid] = sum;
    }
  }

  if (PHASE == 0) {
    // the two halves of a wavefront hold the same query column for different token rows
#pragma unroll
    for (int b = 0; b < 2 * QB; ++b) {
      const float m_o = __shfl_xor(m_run[b], 32, kWave);
      const float l_o = __shfl_xor(l_run[b], 32, kWave);
      const float m_n = fmaxf(m_run[b], m_o);
      const float m_s = (m_n == -INFINITY) ? 0.f : m_n;
      l_run[b] = l_run[b] * ex2(m_run[b] - m_s) + l_o * ex2(m_o - m_s);
      m_run[b] = m_n;
      if (half == 0) sm_stats[wave][b * 32 + col] = make_float2(m_run[b], l_run[b]);
    }
    __syncthreads();
    if (tid < QROWS && qp + tid < R) {
      float M = -INFINITY;
#pragma unroll
      for (int w = 0; w < NW; ++w) M = fmaxf(M, sm_stats[w][tid].x);
      float Z = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float2 s = sm_stats[w][tid];
        if (s.y > 0.f) Z += s.y * ex2(s.x - M);
      }
      stats_part[(part_base + chunk) * R + qp + tid] = make_float2(M, Z);
    }
  }
}

template <int D, bool STREAM, bool CAUSAL, int QB>
hipError_t launch_wide_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                         const int32_t* counts_in, float* alpha_bar, const Workspace& ws, const void* V,
                         hipStream_t stream) {
  dim3 grid(tab.total_chunks), block(QB == 2 ? 256 : 512);
  hipLaunchKernelGGL((score_mfma_wide_kernel<D, 0, STREAM, CAUSAL, false, QB>), grid, block, 0, stream, tab, sh,
                     (const uint16_t*)Q, (const uint16_t*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row,
                     (const uint16_t*)nullptr, (float*)nullptr, 0);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if ((e = launch_score_finalize(tab, sh, ws, stream)) != hipSuccess) return e;
  if (V != nullptr) {
    hipLaunchKernelGGL((score_mfma_wide_kernel<D, 1, STREAM, CAUSAL, true, QB>), grid, block, 0, stream, tab, sh,
                       (const uint16_t*)Q, (const uint16_t*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row,
                       (const uint16_t*)V, ws.o_part, 0);
  } else {
    hipLaunchKernelGGL((score_mfma_wide_kernel<D, 1, STREAM, CAUSAL, false, QB>), grid, block, 0, stream, tab, sh,
                       (const uint16_t*)Q, (const uint16_t*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row,
                       (const uint16_t*)nullptr, (float*)nullptr, 0);
  }
  return hipGetLastError();
}

// More than 256 query rows: one launch of the four-block kernel per 256 rows and sweep.
template <int D, bool STREAM, bool CAUSAL>
hipError_t launch_wide_multi_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                               const int32_t* counts_in, float* alpha_bar, const Workspace& ws, const void* V,
                               hipStream_t stream) {
  dim3 grid(tab.total_chunks), block(512);
  hipError_t e;
  for (int qp = 0; qp < sh.R; qp += 256) {
    hipLaunchKernelGGL((score_mfma_wide_kernel<D, 0, STREAM, CAUSAL, false, 4, true>), grid, block, 0, stream, tab, sh,
                       (const uint16_t*)Q, (const uint16_t*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row,
                       (const uint16_t*)nullptr, (float*)nullptr, qp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if ((e = launch_score_finalize(tab, sh, ws, stream)) != hipSuccess) return e;
  for (int qp = 0; qp < sh.R; qp += 256) {
    const bool last = qp + 256 >= sh.R;
    if (last && V != nullptr) {
      hipLaunchKernelGGL((score_mfma_wide_kernel<D, 1, STREAM, CAUSAL, true, 4, true>), grid, block, 0, stream, tab, sh,
                         (const uint16_t*)Q, (const uint16_t*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row,
                         (const uint16_t*)V, ws.o_part, qp);
    } else {
      hipLaunchKernelGGL((score_mfma_wide_kernel<D, 1, STREAM, CAUSAL, false, 4, true>), grid, block, 0, stream, tab,
                         sh, (const uint16_t*)Q, (const uint16_t*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row,
                         (const uint16_t*)nullptr, (float*)nullptr, qp);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

template <int D>
hipError_t launch_wide_multi(const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                             const int32_t* counts_in, float* alpha_bar, const Workspace& ws, const void* V,
                             hipStream_t stream) {
  if (sh.causal > 0) {
    return sh.stream ? launch_wide_multi_t<D, true, true>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream)
                     : launch_wide_multi_t<D, false, true>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream);
  }
  return sh.stream ? launch_wide_multi_t<D, true, false>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream)
                   : launch_wide_multi_t<D, false, false>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream);
}

template <int D, int QB>
hipError_t launch_wide(const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                       const int32_t* counts_in, float* alpha_bar, const Workspace& ws, const void* V,
                       hipStream_t stream) {
  if (sh.causal > 0) {
    return sh.stream ? launch_wide_t<D, true, true, QB>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream)
                     : launch_wide_t<D, false, true, QB>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream);
  }
  return sh.stream ? launch_wide_t<D, true, false, QB>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream)
                   : launch_wide_t<D, false, false, QB>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream);
}

template <int D, int NT, int WQ>
hipError_t launch_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                    const int32_t* counts_in, float* alpha_bar, const Workspace& ws, hipStream_t stream) {
  dim3 grid(tab.total_chunks), block(kThreads);
  hipLaunchKernelGGL((score_mfma_kernel<D, NT, WQ, 0>), grid, block, 0, stream, tab, sh, (const uint16_t*)Q,
                     (const uint16_t*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if ((e = launch_score_finalize(tab, sh, ws, stream)) != hipSuccess) return e;
  hipLaunchKernelGGL((score_mfma_kernel<D, NT, WQ, 1>), grid, block, 0, stream, tab, sh, (const uint16_t*)Q,
                     (const uint16_t*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row);
  return hipGetLastError();
}

template <int D>
hipError_t launch_d(const UnitTable& tab, const Shape& sh, const void* Q, const void* K,
                    const int32_t* counts_in, float* alpha_bar, const Workspace& ws, const void* V,
                    hipStream_t stream) {
  // At most 64 query rows per wavefront: with more, the stationary Q operands, the accumulators and
  // the tile operands no longer fit the 256 registers that two wavefronts per SIMD leave each, and
  // every spill reload waits for ALL loads in flight, the tile prefetch included.
  const int R = sh.R;
  if (R <= 32) return launch_t<D, 1, 1>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream);
  if (R <= 64) return launch_t<D, 2, 1>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream);
  // 65..256 rows: rows 64.. from LDS, one pass over K (KVS_DEBUG_SCORE_WIDE keeps the kernel below for more than 128)
  const bool wide_off = debug_switch(KVS_DEBUG_SCORE_WIDE) == 1;
  if (R <= 128) return launch_wide<D, 2>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream);
  if (R <= 192 && !wide_off) return launch_wide<D, 3>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream);
  if (R <= 256 && !wide_off) return launch_wide<D, 4>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream);
  if (!wide_off) return launch_wide_multi<D>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream);   // 256 rows per launch
  if (R <= 256) return launch_t<D, 2, 2>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream);    // two passes of 128 rows
  return launch_t<D, 2, 4>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream);                  // passes of 256 rows
}

// ------------------------------------------------------------------------------------------------
// fp32 inputs: the same two sweeps with v_mfma_f32_32x32x2_f32 (full fp32 products and sums).  The contraction
// index is split between the halves of the wavefront (lanes 0..31 take elements 0..D/2-1 of a row, lanes 32..63
// the rest: any split works as long as both operands use the same one), so a lane's operands are D/2 contiguous
// floats of one row.  The K tile (32 rows) goes straight from global memory to registers, the tile after it is
// requested before the products of this one start; the Q block (up to 128 rows per launch, rows qp.. of every
// unit) sits in LDS, XOR-swizzled in 16-byte pieces, and is re-read for every tile.  Accumulator layouts, the
// running statistics of sweep 0, the transposed products of sweep 1 and the row offset qp for windows of more
// than 128 rows are those of score_mfma_wide_kernel.  The work is bound by the fp32 matrix rate, not by memory.
template <int D, int PHASE, bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void score_mfma_f32_kernel(
    const UnitTable tab, const Shape sh, const float* __restrict__ Q, const float* __restrict__ K,
    const int32_t* __restrict__ counts_in, float* __restrict__ alpha_bar, float2* __restrict__ stats_part,
    const float* __restrict__ c_row, const int qp) {
  constexpr int ROWB = D * 4;               // bytes per row
  constexpr int LPR = ROWB / 16;            // 16-byte pieces per row
  constexpr int RPI = kWave / LPR;          // rows per load instruction of the Q block
  constexpr int HALF = D / 2;               // contraction indices per half of the wavefront
  constexpr int NQ4 = HALF / 4;             // 16-byte operand pieces per lane and row
  constexpr int QROWS = 128;                // query rows per launch
  constexpr int NBLK = QROWS / 32;

  __shared__ __attribute__((aligned(1024))) unsigned char sm_q[QROWS * ROWB];
  __shared__ float2 sm_stats[kWaves][QROWS];
  __shared__ __attribute__((aligned(16))) float sm_cq[QROWS];
  __shared__ __attribute__((aligned(16))) int sm_lim[QROWS];

  const int ui = find_unit(tab, blockIdx.x);
  const Unit un = tab.unit(ui);
  const int chunk = blockIdx.x - un.chunk_base;
  const int t0 = chunk * un.chunk_len;
  const int t1 = min(un.len, t0 + un.chunk_len);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int iters = (ntiles + kWaves - 1) / kWaves;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int col = lane % 32, half = lane / 32;
  const int R = sh.R;
  const int rows_here = min(R - qp, QROWS);                 // query rows of this launch
  const float sl2 = sh.scale_log2;
  const int32_t* cnt = counts_in ? counts_in + un.in_row : nullptr;
  const float sc = cnt ? 1.f : sl2;
  const size_t part_base = (size_t)un.index * kMaxChunks;
  const bool last_launch = qp + QROWS >= R;

  const unsigned char* Kg = reinterpret_cast<const unsigned char*>(K + (size_t)un.in_row * D);
  const uint4* Qg = reinterpret_cast<const uint4*>(Q + (size_t)un.index * R * D);

  if (PHASE == 1) {
    if (tid < QROWS) {
      sm_cq[tid] = (qp + tid < R) ? c_row[(size_t)un.index * R + qp + tid] : INFINITY;
      sm_lim[tid] = last_seen_row(CAUSAL ? sh.causal : 0, un.len, qp + tid);
    }
  }
  int lim[NBLK];
#pragma unroll
  for (int b = 0; b < NBLK; ++b) lim[b] = last_seen_row(CAUSAL ? sh.causal : 0, un.len, qp + b * 32 + col);

  // the Q block, once per workgroup: every wavefront fetches 32 rows (rows past R repeat the last one); physical
  // piece s of local row r holds logical piece s ^ (r % LPR)
  {
    const int st_row = lane / LPR, st_slot = lane % LPR;
    constexpr int QLD = 32 / RPI;
#pragma unroll
    for (int i = 0; i < QLD; ++i) {
      const int lr = wave * 32 + i * RPI + st_row;
      const int qrow = min(qp + lr, R - 1);
      const int piece = st_slot ^ (lr % LPR);
      __builtin_amdgcn_global_load_lds(KVS_GLOBAL_PTR(Qg + (size_t)qrow * LPR + piece),
                                       KVS_LDS_PTR(sm_q + (wave * 32 + i * RPI) * ROWB), 16, 0, 0);
    }
  }
  // this lane's operand pieces of Q block row `col` (+ 32 per block): logical piece half * NQ4 + i
  const float4* q_ptr[NQ4];
#pragma unroll
  for (int i = 0; i < NQ4; ++i) {
    q_ptr[i] = reinterpret_cast<const float4*>(sm_q + col * ROWB + (((half * NQ4 + i) ^ (col % LPR)) * 16));
  }
  // K tile of the wavefront's tile j: row `col`, elements half * HALF .. + HALF - 1 (the ragged last tile is moved
  // back to end at the chunk's end, see score_mfma_kernel)
  auto load_tile = [&](int j, float4 (&dst)[NQ4]) {
    const int tile_t0 = t0 + j * kTile;
    if (tile_t0 >= t1) return;
    const int base_t = min(tile_t0, t1 - kTile);
    const float4* src = reinterpret_cast<const float4*>(Kg + (size_t)(base_t + col) * ROWB + half * (HALF * 4));
#pragma unroll
    for (int i = 0; i < NQ4; ++i) dst[i] = src[i];
  };
  float4 a4[NQ4], an4[NQ4];
#pragma unroll
  for (int i = 0; i < NQ4; ++i) { a4[i] = make_float4(0.f, 0.f, 0.f, 0.f); an4[i] = a4[i]; }
  load_tile(wave, a4);
  __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): the Q block has landed in LDS
  __syncthreads();

  float m_run[NBLK], l_run[NBLK];
#pragma unroll
  for (int b = 0; b < NBLK; ++b) { m_run[b] = -INFINITY; l_run[b] = 0.f; }

  for (int it = 0; it < iters; ++it) {
    const int j = it * kWaves + wave;
    const int tile_t0 = t0 + j * kTile;
    if (tile_t0 >= t1) break;                       // this wavefront has run out of tiles
    const int base_t = min(tile_t0, t1 - kTile);
    const int shift = tile_t0 - base_t;             // leading rows that belong to the tile before
    load_tile(j + kWaves, an4);                     // flies during this tile's products
    asm volatile("" ::: "memory");

    float p_tok = 0.f;                              // sweep 1: this lane's token, summed over its query rows
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
      if (b * 32 >= rows_here) break;               // uniform: no such rows in this launch
      f32x16 acc[1];
      acc[0] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < NQ4; ++i) {
        const float4 q4 = *reinterpret_cast<const float4*>(reinterpret_cast<const unsigned char*>(q_ptr[i]) +
                                                           b * 32 * ROWB);
        const float qv[4] = {q4.x, q4.y, q4.z, q4.w};
        const float kv[4] = {a4[i].x, a4[i].y, a4[i].z, a4[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[0] = (PHASE == 0) ? __builtin_amdgcn_mfma_f32_32x32x2f32(kv[e], qv[e], acc[0], 0, 0, 0)
                                : __builtin_amdgcn_mfma_f32_32x32x2f32(qv[e], kv[e], acc[0], 0, 0, 0);
        }
      }
      if (PHASE == 0) {
        // accumulator element v of a lane: token row 8*(v/4) + 4*half + v%4, query column `col`
        if (shift > 0) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v / 4) + 4 * half + (v % 4);
            if (row < shift) acc[0][v] = -INFINITY;
          }
        }
        if (CAUSAL && base_t + kTile > un.len - sh.causal + 1) {
          const int lim1[1] = {lim[b]};
          mask_causal<1>(acc, lim1, base_t, half);
        }
        if (cnt) logits_with_counts<1>(acc, cnt, base_t, half, sl2);
        float tm = acc[0][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tm = fmaxf(tm, acc[0][v]);
        const float m_new = fmaxf(m_run[b], tm * sc);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        float sum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += ex2(fmaf(acc[0][v], sc, -m_safe));
        l_run[b] = l_run[b] * ex2(m_run[b] - m_safe) + sum;
        m_run[b] = m_new;
      } else {
        // products taken as Q K^T: accumulator element v is query row 32 b + 8 (v / 4) + 4 half + v % 4 and the
        // lane's column is ONE token
        const bool tail = CAUSAL && base_t + kTile > un.len - sh.causal + 1;       // uniform
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int q0 = 32 * b + 8 * g + 4 * half;
          const float4 c4 = *reinterpret_cast<const float4*>(&sm_cq[q0]);
          const float cq[4] = {c4.x, c4.y, c4.z, c4.w};
          float e[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) e[i] = ex2(fmaf(acc[0][4 * g + i], sl2, -cq[i]));
          if (tail) {
            const int4 l4 = *reinterpret_cast<const int4*>(&sm_lim[q0]);
            const int lq[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) e[i] = (base_t + col > lq[i]) ? 0.f : e[i];
          }
          p_tok += (e[0] + e[1]) + (e[2] + e[3]);
        }
      }
    }
    if (PHASE == 1) {
      p_tok += __shfl_xor(p_tok, 32, kWave);
      if (qp > 0) p_tok += alpha_bar[un.in_row + base_t + col];              // the rows of the launches before
      if (cnt && last_launch) p_tok *= (float)cnt[base_t + col];
      if (half == 0 && col >= shift) alpha_bar[un.in_row + base_t + col] = p_tok;
    }
#pragma unroll
    for (int i = 0; i < NQ4; ++i) a4[i] = an4[i];
  }

  if (PHASE == 0) {
    // the two halves of a wavefront hold the same query column for different token rows
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
      const float m_o = __shfl_xor(m_run[b], 32, kWave);
      const float l_o = __shfl_xor(l_run[b], 32, kWave);
      const float m_n = fmaxf(m_run[b], m_o);
      const float m_s = (m_n == -INFINITY) ? 0.f : m_n;
      l_run[b] = l_run[b] * ex2(m_run[b] - m_s) + l_o * ex2(m_o - m_s);
      m_run[b] = m_n;
      if (half == 0) sm_stats[wave][b * 32 + col] = make_float2(m_run[b], l_run[b]);
    }
    __syncthreads();
    if (tid < rows_here) {
      float M = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sm_stats[w][tid].x);
      float Z = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float2 st = sm_stats[w][tid];
        if (st.y > 0.f) Z += st.y * ex2(st.x - M);
      }
      stats_part[(part_base + chunk) * R + qp + tid] = make_float2(M, Z);
    }
  }
}

template <int D, bool CAUSAL>
hipError_t launch_f32_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const int32_t* counts_in,
                        float* alpha_bar, const Workspace& ws, hipStream_t stream) {
  dim3 grid(tab.total_chunks), block(kThreads);
  hipError_t e;
  for (int qp = 0; qp < sh.R; qp += 128) {
    hipLaunchKernelGGL((score_mfma_f32_kernel<D, 0, CAUSAL>), grid, block, 0, stream, tab, sh, (const float*)Q,
                       (const float*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row, qp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if ((e = launch_score_finalize(tab, sh, ws, stream)) != hipSuccess) return e;
  for (int qp = 0; qp < sh.R; qp += 128) {
    hipLaunchKernelGGL((score_mfma_f32_kernel<D, 1, CAUSAL>), grid, block, 0, stream, tab, sh, (const float*)Q,
                       (const float*)K, counts_in, alpha_bar, ws.stats_part, ws.c_row, qp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

template <int D>
hipError_t launch_f32(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const int32_t* counts_in,
                      float* alpha_bar, const Workspace& ws, hipStream_t stream) {
  return sh.causal > 0 ? launch_f32_t<D, true>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream)
                       : launch_f32_t<D, false>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream);
}

}  // namespace

// One to three query rows stay with the vector kernels (a dot product per row and token keeps up with memory
// there); from four rows on a padded block of 32 on the matrix cores is faster (measured at 8 rows, 32 units of
// 32768 tokens, bf16: 260 against 420 us for the step).
bool score_mfma_supported(const UnitTable& tab, const Shape& sh, kvs_dtype dt) {
  (void)dt;
  if (sh.R < 4) return false;
  for (int i = 0; i < tab.n_units; ++i) {
    if (tab.unit(i).len < kTile) return false;   // the tile loads assume 32 whole rows per unit
  }
  return true;
}

// Sweep 1 of the kernel for more than 64 query rows can carry the pass over V along (o_part then holds one partial
// per score chunk).
bool score_mfma_takes_values(const Shape& sh, kvs_dtype dt) {
  if (dt != KVS_BF16) return false;
  const bool wide_off = debug_switch(KVS_DEBUG_SCORE_WIDE) == 1;
  return sh.R > 64 && (sh.R <= 128 || !wide_off);
}

// V: non-null asks for that fused pass (only where score_mfma_takes_values says so).
hipError_t launch_score_mfma(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* Q, const void* K,
                             const int32_t* counts_in, float* alpha_bar, const Workspace& ws, const void* V,
                             hipStream_t stream) {
  if (dt == KVS_F32) {
    return sh.D == 64 ? launch_f32<64>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream)
                      : launch_f32<128>(tab, sh, Q, K, counts_in, alpha_bar, ws, stream);
  }
  return sh.D == 64 ? launch_d<64>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream)
                    : launch_d<128>(tab, sh, Q, K, counts_in, alpha_bar, ws, V, stream);
}

}  // namespace kvs
