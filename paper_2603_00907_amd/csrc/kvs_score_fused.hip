// One-pass score kernel (bf16, windows of 65..128 query rows): K is read from memory ONCE.
//
// Sec. 4.1, Eq. attn_def_vec needs every logit twice: once for the softmax normaliser of its query row (a
// reduction over ALL cached Keys), once for the normalised weight that is averaged over the rows into alpha_bar.
// Nothing in it needs K twice, as long as the Keys can wait on chip for the normalisers.  A work item is a chunk of
// kFusedChunkBytes of K rows (512 tokens at head_dim 128), which one workgroup of eight wavefronts (one per CU)
// keeps in LDS for the item's whole life:
//   A  the chunk streams into LDS (global_load_lds, XOR-swizzled, a 32-token tile per group of instructions); every
//      wavefront takes its tiles as they land, computes S^T = K_tile Q^T with v_mfma_f32_32x32x16_bf16 and the
//      running (maximum, sum of exponentials) of the 128 query columns; the workgroup publishes, per query row,
//      log2 of the chunk's sum of 2^logit;
//   -  it waits until every chunk of its unit has published: the workgroup that publishes last reduces the unit's
//      chunk values to one normaliser per query row, c[q] = log2(R sum_t 2^logit), and writes them out;
//   B  the logits are recomputed from the chunk that is still in LDS (as Q K^T: a lane holds one token, the sum over
//      the query rows is a sum over registers), alpha_bar leaves, and the pass over V rides along
//      (o_bar = sum_t alpha_bar[t] V[t]; one partial sum per work item).
// The time from the first load of an item to the end of its phase B is what bounds the kernel (the LDS of the chip
// holds 32 MB of K at a time), so the path between the phases is kept short: the normalisers are marked words that
// the waiting workgroups poll directly (no flag, no second round trip), the reduction is one batch of loads.
//
// Work items are handed out by an atomic ticket counter in unit order to a grid of persistent workgroups, so a
// taken item always belongs to a workgroup that is running, and a running workgroup publishes its item's
// statistics before it waits for anything: no workgroup ever waits for work that has not started.  Every wait is
// bounded all the same (a time limit and a poll limit): a workgroup whose unit is not complete in time (few
// workgroups resident, e.g. beside other kernels), or whose unit is so long that its last chunks cannot start
// while this one is held, puts its item on a list and goes on; a second, ordinary kernel (this one with
// SECOND = true) redoes phase B for the listed items from memory, after the first has ended and all normalisers
// are final.  Nothing spins forever whatever the residency.
//
// Cross-workgroup data (chunk values, normalisers, counters) moves with agent-scope atomic loads and stores, which
// pass the per-XCD L2 caches; a publisher waits for its stores' completion before it bumps the unit's counter.  No
// fence instruction (an L2 write-back on this chip) is used.
#include <type_traits>

#include "kvs_mfma_tile.h"

namespace kvs {
namespace {

using namespace mfma;

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;
constexpr unsigned kMaxPolls = 1u << 16;    // second bound on a wait, should the clock ever misbehave
constexpr int kQRows = 128;                 // query rows per workgroup (two blocks of 64)

template <int N>
__device__ __forceinline__ void wait_vm() {   // at most N vector-memory operations still in flight
  static_assert(N >= 0 && N < 64, "vmcnt is six bits");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  asm volatile("" ::: "memory");
}
// (the counts are multiples of a tile's load instructions; k is uniform)
template <int NLD>
__device__ __forceinline__ void wait_tiles_in_flight(int k) {
  if (k <= 0) wait_vm<0>();
  else if (k == 1) wait_vm<NLD>();
  else if (k == 2) wait_vm<2 * NLD>();
  else if (k == 3) wait_vm<3 * NLD>();
  else wait_vm<4 * NLD>();
}

// Operand reads of one pair of k-steps, complete on return (inline assembly for the reason given at lds_read_4x16):
// the K tile's two pieces at a0, a1 (+ OFFA), and for the query rows kept in LDS their pieces at q0, q1 and 32 rows
// further.
template <int OFFA>
__device__ __forceinline__ void lds_read_a2(bf16x8& a0, bf16x8& a1, uint32_t ad0, uint32_t ad1) {
  asm volatile(
      "ds_read_b128 %0, %2 offset:%4\n\t"
      "ds_read_b128 %1, %3 offset:%4\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(a0), "=&v"(a1)
      : "v"(ad0), "v"(ad1), "n"(OFFA)
      : "memory");
}
template <int OFFA, int OFFQ1>
__device__ __forceinline__ void lds_read_a2_q4(bf16x8& a0, bf16x8& a1, bf16x8& b00, bf16x8& b01, bf16x8& b10,
                                               bf16x8& b11, uint32_t ad0, uint32_t ad1, uint32_t q0, uint32_t q1) {
  asm volatile(
      "ds_read_b128 %0, %6 offset:%10\n\t"
      "ds_read_b128 %1, %7 offset:%10\n\t"
      "ds_read_b128 %2, %8\n\t"
      "ds_read_b128 %3, %8 offset:%11\n\t"
      "ds_read_b128 %4, %9\n\t"
      "ds_read_b128 %5, %9 offset:%11\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(a0), "=&v"(a1), "=&v"(b00), "=&v"(b01), "=&v"(b10), "=&v"(b11)
      : "v"(ad0), "v"(ad1), "v"(q0), "v"(q1), "n"(OFFA), "n"(OFFQ1)
      : "memory");
}

__device__ __forceinline__ unsigned ld_agent(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(unsigned* p, unsigned v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent_f(const float* p) {
  return __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned*>(p), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void st_agent_f(float* p, float v) {
  __hip_atomic_store(reinterpret_cast<unsigned*>(p), __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// log2(2^a + 2^b) (either may be -inf)
__device__ __forceinline__ float lse2(float a, float b) {
  const float m = fmaxf(a, b);
  if (m == -INFINITY) return m;
  return m + __builtin_amdgcn_logf(ex2(a - m) + ex2(b - m));
}

// Before the one-pass kernel: counters to zero, the launch's normalisers to "not yet" (one block per unit).
__global__ void score_fused_init_kernel(const UnitTable tab, const int R, float* c_row, unsigned int* fsync,
                                        unsigned int* sel_shared) {
  const Unit un = tab.unit(blockIdx.x);
  if (sel_shared != nullptr && blockIdx.x < kInlineUnits) {   // the exchange area of the selection that follows starts from zero
    uint4* z = reinterpret_cast<uint4*>(sel_shared + (size_t)blockIdx.x * kSelSharedInts);
    for (int i = threadIdx.x; i < kSelSharedInts / 4; i += blockDim.x) z[i] = make_uint4(0u, 0u, 0u, 0u);
  }
  for (int q = threadIdx.x; q < R; q += blockDim.x) {
    reinterpret_cast<unsigned int*>(c_row)[(size_t)un.index * R + q] = kFusedNotYet;
  }
  if (blockIdx.x == 0 && threadIdx.x < kFusedSyncInts) fsync[threadIdx.x] = 0u;
}

template <int D, bool STREAM, bool CAUSAL, bool SECOND>
__global__ __launch_bounds__(kThreads, 1) void score_fused_kernel(
    const UnitTable tab, const Shape sh, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, const int32_t* __restrict__ counts_in, float* __restrict__ alpha_bar,
    float* fstats, float* c_row, float* __restrict__ fo_part, unsigned int* fsync, const unsigned timeout_ticks,
    const unsigned stagger_ticks) {
  constexpr int KS = D / 16;                // MFMA k-steps per tile
  constexpr int LPR = D / 8;                // 16-byte pieces (= lanes) per row
  constexpr int RPI = kWave / LPR;          // rows per load instruction
  constexpr int NLD = kTile / RPI;          // load instructions per tile
  constexpr int ROWB = D * 2;
  constexpr int TILEB = kTile * ROWB;
  constexpr int NT_CH = kFusedChunkBytes / TILEB;            // tiles per work item
  constexpr int CH = NT_CH * kTile;                          // tokens per work item
  constexpr int MAXT = NT_CH / kWaves;                       // tiles per wavefront: tiles w MAXT .. w MAXT + MAXT - 1
  static_assert(KS == 4 || KS == 8, "k-steps come in pairs");
  static_assert(NT_CH % kWaves == 0 && MAXT <= 4, "wait_tiles_in_flight");
  static_assert((MAXT - 1) * TILEB < 65536, "tile offsets are ds_read immediates");

  __shared__ __attribute__((aligned(1024))) unsigned char sm_k[NT_CH * TILEB];
  __shared__ __attribute__((aligned(1024))) unsigned char sm_q[64 * ROWB];     // query rows 64..127
  __shared__ __attribute__((aligned(16))) float sm_lse[kWaves][kQRows];        // also: finalize pairs, o_bar sums
  __shared__ __attribute__((aligned(16))) float sm_cq[kQRows];
  __shared__ __attribute__((aligned(16))) int sm_lim[kQRows];
  __shared__ unsigned sm_item;
  __shared__ int sm_last, sm_fail;

  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int col = lane % 32, half = lane / 32;
  const int R = sh.R;
  const float sl2 = sh.scale_log2;
  const int st_row = lane / LPR, st_slot = lane % LPR;

  int ld_off[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int row = st_row + i * RPI;
    ld_off[i] = row * ROWB + (st_slot ^ (row % LPR)) * 16;
  }
  // LDS byte addresses of this lane's operand pieces: row `col` of the wavefront's first tile
  uint32_t a_addr[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    const uint32_t off = col * ROWB + ((2 * kk + half) ^ (col % LPR)) * 16;
    a_addr[kk] = (uint32_t)(size_t)KVS_LDS_PTR(sm_k) + wave * MAXT * TILEB + off;
  }
  // (the same piece of row `col` of sm_q lies q_delta bytes further: one address array serves both)
  const uint32_t q_delta =
      (uint32_t)(size_t)KVS_LDS_PTR(sm_q) - (uint32_t)(size_t)KVS_LDS_PTR(sm_k) - wave * MAXT * TILEB;
  unsigned int* const done = fsync + kFusedDone;
  unsigned int* const deferred = fsync + kFusedSyncInts;
  unsigned int* const c_bits = reinterpret_cast<unsigned int*>(c_row);
  const unsigned total = (unsigned)tab.total_fitems;
  const unsigned n_second = SECOND ? min(fsync[kFusedDeferred], total) : 0u;
  unsigned second_pos = blockIdx.x;

#ifdef KVS_FUSED_PROFILE
  unsigned long long pf_t = 0, pf_a = 0, pf_w = 0, pf_f = 0, pf_b = 0, pf_q = 0;
  unsigned pf_items = 0, pf_last = 0;
#define PF_MARK(acc) do { if (tid == 0) { const unsigned long long now_ = wall_clock64(); acc += now_ - pf_t; pf_t = now_; } } while (0)
#else
#define PF_MARK(acc) do { } while (0)
#endif
  int have_unit = -1;                       // the unit whose Q block this workgroup holds
  bf16x8 bq[2][KS];                         // query rows 0..63, register-stationary
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // The workgroups start in four cohorts, a fraction of an item's life apart: workgroups that start together go
  // through their items' phases together (all of them wait for the same units), and four cohorts out of step keep
  // loads, arithmetic and waits of different workgroups on the chip at the same time.
  if (!SECOND && stagger_ticks > 0) {
    const unsigned cohort = (4u * blockIdx.x) / gridDim.x;
    const unsigned long long t_go = wall_clock64() + (unsigned long long)cohort * stagger_ticks;
    for (unsigned poll = 0; poll < kMaxPolls && wall_clock64() < t_go; ++poll) __builtin_amdgcn_s_sleep(16);
  }
  // the ticket of the next item is taken while the current item's phase B runs (thread 0 holds it)
  unsigned next_item = 0;
  if (!SECOND && tid == 0) {
    next_item = __hip_atomic_fetch_add(&fsync[kFusedTicket], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  for (;;) {
    // ---- the next work item (the barrier also ends every use of the shared tables by the item before)
    unsigned item;
    if (SECOND) {
      __syncthreads();
      if (second_pos >= n_second) break;
      item = deferred[second_pos];
      second_pos += gridDim.x;
      if (item >= total) continue;           // cannot happen: the first kernel lists items it was given
    } else {
      if (tid == 0) { sm_item = next_item; sm_fail = 0; }
      __syncthreads();
      item = sm_item;
    }
    item = (unsigned)__builtin_amdgcn_readfirstlane((int)item);
    if (item >= total) break;
#ifdef KVS_FUSED_PROFILE
    if (tid == 0) { pf_t = wall_clock64(); ++pf_items; }
#endif
    const int ui = find_unit_by<&Unit::f_base>(tab, (int)item);
    const Unit un = tab.unit(ui);
    const int chunk = (int)item - un.f_base;
    const int n_chunks = fused_chunks(un.len, D);
    const int t0 = chunk * CH;
    const int t1 = min(un.len, t0 + CH);
    const int ntiles = (t1 - t0 + kTile - 1) / kTile;
    const int ntw = min(max(ntiles - wave * MAXT, 0), MAXT);                 // this wavefront's tiles
    const int32_t* cnt = counts_in ? counts_in + un.in_row : nullptr;
    const float sc = cnt ? 1.f : sl2;        // the accumulators hold finished logits when cardinalities were added
    const unsigned char* Kg = reinterpret_cast<const unsigned char*>(K + (size_t)un.in_row * D);
    const unsigned char* Vg = reinterpret_cast<const unsigned char*>(V + (size_t)un.in_row * D);

    // ---- the unit's Q block when it is not the one already held: rows 64..127 to LDS, rows 0..63 to registers in
    //      operand order (a lane's 16-byte pieces of its own row; 16 KB from L2 per item at most)
    const bool new_q = un.index != have_unit;
    if (new_q) {
      const uint16_t* Qu = Q + (size_t)un.index * R * D;
      const uint4* Qg = reinterpret_cast<const uint4*>(Qu);
      constexpr int RPW = 64 / kWaves;         // rows of sm_q per wavefront
      constexpr int QLD = RPW / RPI;
      static_assert(RPW % RPI == 0 && QLD >= 1, "whole load instructions");
#pragma unroll
      for (int i = 0; i < QLD; ++i) {
        const int lr = wave * RPW + i * RPI + st_row;
        const int qrow = min(64 + lr, R - 1);                       // rows past R repeat the last one
        const int piece = st_slot ^ (lr % LPR);
        __builtin_amdgcn_global_load_lds(KVS_GLOBAL_PTR(Qg + (size_t)qrow * LPR + piece),
                                         KVS_LDS_PTR(sm_q + (wave * RPW + i * RPI) * ROWB), 16, 0, 0);
      }
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const int qrow = min(nt * 32 + col, R - 1);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
          const uint4 raw = *reinterpret_cast<const uint4*>(Qu + (size_t)qrow * D + kk * 16 + 8 * half);
          bq[nt][kk] = *reinterpret_cast<const bf16x8*>(&raw);
        }
      }
      have_unit = un.index;
    }
    // ---- the item's K tiles: tile j of the chunk goes to buffer j, wavefront w takes tiles w MAXT ...
    //      (the ragged last tile is moved back so that it ends at the chunk's end; the rows it shares with the
    //      tile before are masked out below; every unit has at least 32 rows on this path)
#pragma unroll
    for (int jj = 0; jj < MAXT; ++jj) {
      if (jj < ntw) {
        const int j = wave * MAXT + jj;
        const int base_t = min(t0 + j * kTile, t1 - kTile);
        const unsigned char* base = Kg + (size_t)base_t * ROWB;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          __builtin_amdgcn_global_load_lds(KVS_GLOBAL_PTR(base + ld_off[i]),
                                           KVS_LDS_PTR(sm_k + j * TILEB + i * 1024), 16, 0, STREAM ? kNonTemporal : 0);
        }
      }
    }
    if (new_q) {                               // loads return in order: the Q block is there when only K tiles fly
      wait_tiles_in_flight<NLD>(ntw);
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    }

    // One block of 64 query rows (h = 0: rows 0..63 from registers, h = 1: rows 64..127 from sm_q) against tile JJ
    // of this wavefront, whose operand pieces are read from LDS pair by pair of k-steps (the tile stays there
    // anyway, so nothing of it is held in registers).  ORIENT 0: S^T = K Q^T (a lane holds one query column),
    // 1: S = Q K^T (a lane holds one token).
    auto products = [&](auto hc, auto oc, auto jc, f32x16 (&acc)[2]) {
      constexpr int h = decltype(hc)::value;
      constexpr int ORIENT = decltype(oc)::value;
      constexpr int OFFA = decltype(jc)::value * TILEB;
#pragma unroll
      for (int kp = 0; kp < KS / 2; ++kp) {
        bf16x8 a0, a1, b00, b01, b10, b11;
        if (h == 0) {
          lds_read_a2<OFFA>(a0, a1, a_addr[2 * kp], a_addr[2 * kp + 1]);
          b00 = bq[0][2 * kp]; b01 = bq[1][2 * kp]; b10 = bq[0][2 * kp + 1]; b11 = bq[1][2 * kp + 1];
        } else {
          lds_read_a2_q4<OFFA, 32 * ROWB>(a0, a1, b00, b01, b10, b11, a_addr[2 * kp], a_addr[2 * kp + 1],
                                          a_addr[2 * kp] + q_delta, a_addr[2 * kp + 1] + q_delta);
        }
        if (ORIENT == 0) {
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b00, kp == 0 ? zero : acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b01, kp == 0 ? zero : acc[1], 0, 0, 0);
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b10, acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b11, acc[1], 0, 0, 0);
        } else {
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b00, a0, kp == 0 ? zero : acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b01, a0, kp == 0 ? zero : acc[1], 0, 0, 0);
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b10, a1, acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b11, a1, acc[1], 0, 0, 0);
        }
      }
    };
    typedef std::integral_constant<int, 0> c0_t;
    typedef std::integral_constant<int, 1> c1_t;
    // a tile's Value rows, RPI whole rows per load
    auto load_values = [&](int jj, u32x4 (&vr)[NLD]) {
      const int base_t = min(t0 + (wave * MAXT + jj) * kTile, t1 - kTile);
      const unsigned char* vt = Vg + (size_t)base_t * ROWB + lane * 16;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const u32x4* src = reinterpret_cast<const u32x4*>(vt + i * 1024);
        vr[i] = STREAM ? __builtin_nontemporal_load(src) : *src;
      }
    };

    PF_MARK(pf_q);
    if (!SECOND) {
      // ---- phase A: running (maximum, sum of exponentials) of this lane's four query columns over its tiles
      float m_run[4], l_run[4];
      int lim[4];                              // causal window: last row each of the lane's query columns attends to
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        m_run[b] = -INFINITY;
        l_run[b] = 0.f;
        lim[b] = last_seen_row(CAUSAL ? sh.causal : 0, un.len, b * 32 + col);
      }
      auto tile_a = [&](auto jc) {
        constexpr int JJ = decltype(jc)::value;
        const int tile_t0 = t0 + (wave * MAXT + JJ) * kTile;
        const int base_t = min(tile_t0, t1 - kTile);
        const int shift = tile_t0 - base_t;          // leading rows that belong to the tile before
        auto stats = [&](auto hc) {
          constexpr int h = decltype(hc)::value;
          f32x16 acc[2];
          products(hc, c0_t{}, jc, acc);
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
          for (int nt = 0; nt < 2; ++nt) {
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
        };
        stats(c0_t{});
        __builtin_amdgcn_sched_barrier(0);
        stats(c1_t{});
      };
      if (0 < ntw) { wait_tiles_in_flight<NLD>(ntw - 1); tile_a(std::integral_constant<int, 0>{}); }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (MAXT > 1) { if (1 < ntw) { wait_tiles_in_flight<NLD>(ntw - 2); tile_a(std::integral_constant<int, 1>{}); } }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (MAXT > 2) { if (2 < ntw) { wait_tiles_in_flight<NLD>(ntw - 3); tile_a(std::integral_constant<int, 2>{}); } }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (MAXT > 3) { if (3 < ntw) { wait_tiles_in_flight<NLD>(ntw - 4); tile_a(std::integral_constant<int, 3>{}); } }
      __builtin_amdgcn_sched_barrier(0);

      // the two halves of a wavefront hold the same query column for different token rows; per column the
      // wavefront leaves log2 of its sum of 2^logit
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const float m_o = __shfl_xor(m_run[b], 32, kWave);
        const float l_o = __shfl_xor(l_run[b], 32, kWave);
        const float m_n = fmaxf(m_run[b], m_o);
        const float m_s = (m_n == -INFINITY) ? 0.f : m_n;
        const float l_n = l_run[b] * ex2(m_run[b] - m_s) + l_o * ex2(m_o - m_s);
        if (half == 0) sm_lse[wave][b * 32 + col] = (l_n > 0.f) ? m_n + __builtin_amdgcn_logf(l_n) : -INFINITY;
      }
      __syncthreads();
      // ---- publish the chunk's values; the stores have completed before the unit's counter moves
      if (tid < kQRows && tid < R) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sm_lse[w][tid]);
        // (a query row that the causal mask cuts off from every token of this item has no finite value here:
        // its share is log2 0)
        float lse = -INFINITY;
        if (M != -INFINITY) {
          float S = 0.f;
#pragma unroll
          for (int w = 0; w < kWaves; ++w) S += ex2(sm_lse[w][tid] - M);    // 2^(-inf) = 0
          lse = M + __builtin_amdgcn_logf(S);
        }
        st_agent_f(&fstats[(size_t)item * R + tid], lse);
      }
      if (tid < kQRows) wait_vm<0>();
      __syncthreads();
      if (tid == 0) {
        const unsigned before = __hip_atomic_fetch_add(&done[ui], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sm_last = (before + 1u == (unsigned)n_chunks);
      }
      __syncthreads();
      PF_MARK(pf_a);
      if (sm_last) {
        // ---- this workgroup published last: the unit's normalisers c[q] = log2(R sum_t 2^logit) from the chunks'
        //      values, in a fixed order (thread (q, h) takes the chunks c = h, h + 4, ...), one batch of loads for
        //      up to 64 chunks
        constexpr int NH = kThreads / kQRows;
        const int q = tid % kQRows, h = tid / kQRows;
        float M = -INFINITY, S = 0.f;
        if (q < R) {
          const float* src = fstats + (size_t)un.f_base * R + q;
          constexpr int UN = 16;
          for (int c0 = h; c0 < n_chunks; c0 += NH * UN) {
            float v[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
              const int c = c0 + NH * u;
              v[u] = -INFINITY;
              if (c < n_chunks) v[u] = ld_agent_f(src + (size_t)c * R);
            }
            float Mn = M;
#pragma unroll
            for (int u = 0; u < UN; ++u) Mn = fmaxf(Mn, v[u]);
            if (Mn != -INFINITY) {
              float add = 0.f;
#pragma unroll
              for (int u = 0; u < UN; ++u) add += ex2(v[u] - Mn);
              S = S * ex2(M - Mn) + add;
              M = Mn;
            }
          }
        }
        float2* sm_pair = reinterpret_cast<float2*>(&sm_lse[0][0]);       // [NH][kQRows]: the wavefronts' table is idle
        sm_pair[h * kQRows + q] = make_float2(M, S);
        __syncthreads();
        if (h == 0) {
          float Mq = -INFINITY;
#pragma unroll
          for (int g = 0; g < NH; ++g) Mq = fmaxf(Mq, sm_pair[g * kQRows + q].x);
          float Sq = 0.f;
#pragma unroll
          for (int g = 0; g < NH; ++g) {
            const float2 p2 = sm_pair[g * kQRows + q];
            if (p2.y > 0.f) Sq += p2.y * ex2(p2.x - Mq);
          }
          const float cq = Mq + __builtin_amdgcn_logf(Sq * (float)R);
          if (q < R) st_agent_f(&c_row[(size_t)un.index * R + q], cq);
          sm_cq[q] = (q < R) ? cq : INFINITY;
        }
        PF_MARK(pf_f);
#ifdef KVS_FUSED_PROFILE
        if (tid == 0) ++pf_last;
#endif
      } else {
        // ---- wait (bounded) for the unit's normalisers: thread q polls its own word.  An item whose unit still has
        //      more chunks to come than half the grid can take is not held: those chunks cannot all start before
        //      this workgroup lets go
        if (tid < kQRows) {
          float cq = INFINITY;
          if (tid < R) {
            bool ok = false;
            if (n_chunks - 1 - chunk <= (int)gridDim.x / 2) {
              const unsigned int* word = c_bits + (size_t)un.index * R + tid;
              const unsigned long long t_start = wall_clock64();
              for (unsigned poll = 0; poll < kMaxPolls; ++poll) {
                const unsigned bits = ld_agent(word);
                if (bits != kFusedNotYet) { cq = __uint_as_float(bits); ok = true; break; }
                if (wall_clock64() - t_start >= (unsigned long long)timeout_ticks) break;
                __builtin_amdgcn_s_sleep(2);
              }
            }
            if (!ok) sm_fail = 1;
          }
          sm_cq[tid] = cq;
        }
        PF_MARK(pf_w);
      }
    } else {
      if (tid < kQRows) sm_cq[tid] = (tid < R) ? c_row[(size_t)un.index * R + tid] : INFINITY;
    }
    if (CAUSAL && tid < kQRows) sm_lim[tid] = last_seen_row(sh.causal, un.len, tid);
    __syncthreads();
    if (!SECOND) {
      if (sm_fail) {                             // (uniform) the second kernel finishes this item
        if (tid == 0) {
          const unsigned pos = __hip_atomic_fetch_add(&fsync[kFusedDeferred], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (pos < total) deferred[pos] = item;
          next_item = __hip_atomic_fetch_add(&fsync[kFusedTicket], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        continue;
      }
      if (tid == 0) {
        next_item = __hip_atomic_fetch_add(&fsync[kFusedTicket], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }

    // ---- phase B: alpha_bar of the item's tokens from the tiles in LDS, and the item's share of o_bar.  A tile's
    //      Value rows are requested before the tile's products and used when its alpha_bar values exist.
    float o_acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o_acc[e] = 0.f;
    auto tile_b = [&](auto jc, const u32x4 (&vr)[NLD]) {
      constexpr int JJ = decltype(jc)::value;
      const int tile_t0 = t0 + (wave * MAXT + JJ) * kTile;
      const int base_t = min(tile_t0, t1 - kTile);
      const int shift = tile_t0 - base_t;
      float p_tok = 0.f;                         // this lane's token, summed over its query rows
      const bool tail = CAUSAL && base_t + kTile > un.len - sh.causal + 1;       // uniform
      auto weights = [&](auto hc) {
        constexpr int h = decltype(hc)::value;
        f32x16 acc[2];
        products(hc, c1_t{}, jc, acc);
        // accumulator element v of block nt: query row 32 (2 h + nt) + 8 (v / 4) + 4 half + v % 4, column = token
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
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
      };
      weights(c0_t{});
      __builtin_amdgcn_sched_barrier(0);
      weights(c1_t{});
      // the two halves of the wavefront hold the token's other query rows; a row that stands for c tokens has c
      // equal terms in every softmax sum (2^(e + log2 c) = c 2^e)
      p_tok += __shfl_xor(p_tok, 32, kWave);
      // lane l holds the weight of tile row l % 32; load i of this lane is row i * RPI + st_row
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int row = i * RPI + st_row;
        float w = __shfl(p_tok, row, kWave);
        if (row < shift) w = 0.f;                           // the tile before has counted this row
        float vf[8];
        Piece<uint16_t>::unpack(make_uint4(vr[i].x, vr[i].y, vr[i].z, vr[i].w), vf);
#pragma unroll
        for (int e = 0; e < 8; ++e) o_acc[e] = fmaf(w, vf[e], o_acc[e]);
      }
      if (cnt) p_tok *= (float)cnt[base_t + col];
      if (half == 0 && col >= shift) alpha_bar[un.in_row + base_t + col] = p_tok;
    };
    __builtin_amdgcn_sched_barrier(0);
    if (0 < ntw) { u32x4 vr[NLD]; load_values(0, vr); tile_b(std::integral_constant<int, 0>{}, vr); }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (MAXT > 1) { if (1 < ntw) { u32x4 vr[NLD]; load_values(1, vr); tile_b(std::integral_constant<int, 1>{}, vr); } }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (MAXT > 2) { if (2 < ntw) { u32x4 vr[NLD]; load_values(2, vr); tile_b(std::integral_constant<int, 2>{}, vr); } }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (MAXT > 3) { if (3 < ntw) { u32x4 vr[NLD]; load_values(3, vr); tile_b(std::integral_constant<int, 3>{}, vr); } }
    __builtin_amdgcn_sched_barrier(0);

    // the item's partial o_bar: lanes that hold the same piece of the row, then the wavefronts, in a fixed order
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
      for (int e = 0; e < 8; ++e) o_acc[e] += __shfl_xor(o_acc[e], off, kWave);
    }
    float* sm_o = &sm_lse[0][0];                                      // (idle between the phases' uses)
    if (st_row == 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) sm_o[wave * D + st_slot * 8 + e] = o_acc[e];
    }
    __syncthreads();
    if (tid < D) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) sum += sm_o[w * D + tid];
      fo_part[(size_t)item * D + tid] = sum;
    }
    PF_MARK(pf_b);
  }
#ifdef KVS_FUSED_PROFILE
  if (!SECOND && tid == 0) {
    // sums over the workgroups, in ticks of 10 ns: Q block + tile issue, phase A + publish, wait, finalize, phase B
    atomicAdd(&fsync[8], (unsigned)pf_q); atomicAdd(&fsync[9], (unsigned)pf_a); atomicAdd(&fsync[10], (unsigned)pf_w);
    atomicAdd(&fsync[11], (unsigned)pf_f); atomicAdd(&fsync[12], (unsigned)pf_b); atomicAdd(&fsync[13], pf_items);
    atomicAdd(&fsync[14], pf_last);
  }
#endif
}

template <int D, bool STREAM, bool CAUSAL>
hipError_t launch_fused_t(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                          const int32_t* counts_in, float* alpha_bar, const Workspace& ws, hipStream_t stream,
                          int grid_first, int grid_second, unsigned timeout_ticks, unsigned stagger_ticks) {
  hipLaunchKernelGGL(score_fused_init_kernel, dim3(tab.n_units), dim3(kQRows), 0, stream, tab, sh.R, ws.c_row, ws.fsync,
                     ws.sel_shared);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((score_fused_kernel<D, STREAM, CAUSAL, false>), dim3(grid_first), dim3(kThreads), 0, stream, tab,
                     sh, (const uint16_t*)Q, (const uint16_t*)K, (const uint16_t*)V, counts_in, alpha_bar, ws.fstats,
                     ws.c_row, ws.fo_part, ws.fsync, timeout_ticks, stagger_ticks);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((score_fused_kernel<D, STREAM, CAUSAL, true>), dim3(grid_second), dim3(kThreads), 0, stream, tab,
                     sh, (const uint16_t*)Q, (const uint16_t*)K, (const uint16_t*)V, counts_in, alpha_bar, ws.fstats,
                     ws.c_row, ws.fo_part, ws.fsync, timeout_ticks, 0u);
  return hipGetLastError();
}

template <int D>
hipError_t launch_fused_d(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                          const int32_t* counts_in, float* alpha_bar, const Workspace& ws, hipStream_t stream,
                          int g1, int g2, unsigned tt, unsigned st) {
  if (sh.causal > 0) {
    return sh.stream ? launch_fused_t<D, true, true>(tab, sh, Q, K, V, counts_in, alpha_bar, ws, stream, g1, g2, tt, st)
                     : launch_fused_t<D, false, true>(tab, sh, Q, K, V, counts_in, alpha_bar, ws, stream, g1, g2, tt, st);
  }
  return sh.stream ? launch_fused_t<D, true, false>(tab, sh, Q, K, V, counts_in, alpha_bar, ws, stream, g1, g2, tt, st)
                   : launch_fused_t<D, false, false>(tab, sh, Q, K, V, counts_in, alpha_bar, ws, stream, g1, g2, tt, st);
}

}  // namespace

bool score_fused_supported(const UnitTable& tab, const Shape& sh, kvs_dtype dt) {
  if (dt != KVS_BF16 || sh.R <= 64 || sh.R > kQRows) return false;
  for (int i = 0; i < tab.n_units; ++i) {
    if (tab.unit(i).len < kTile) return false;   // the tile loads assume 32 whole rows per unit
  }
  return true;
}

hipError_t launch_score_fused(const UnitTable& tab, const Shape& sh, const void* Q, const void* K, const void* V,
                              const int32_t* counts_in, float* alpha_bar, const Workspace& ws, hipStream_t stream) {
  // one persistent workgroup per CU (its LDS holds one), fewer when there are fewer items
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) {
      n_cu = v;
    } else {
      (void)hipGetLastError();
      n_cu = 256;
    }
  }
  const int g1 = std::max(1, std::min(tab.total_fitems, n_cu));
  const int g2 = std::max(1, std::min(tab.total_fitems, n_cu));
  // the clock of wall_clock64() runs at 100 MHz; the switch holds microseconds + 1 (0: the default)
  const int sw = debug_switch(KVS_DEBUG_FUSED_WAIT_US);
  const unsigned ticks = 100u * (unsigned)(sw > 0 ? sw - 1 : 200);
  // cohorts start this many microseconds apart (switch: tenths of a microsecond + 1; 0: the default)
  const int ss = debug_switch(KVS_DEBUG_FUSED_STAGGER);
  const unsigned stagger = 10u * (unsigned)(ss > 0 ? ss - 1 : 0);
  return sh.D == 64 ? launch_fused_d<64>(tab, sh, Q, K, V, counts_in, alpha_bar, ws, stream, g1, g2, ticks, stagger)
                    : launch_fused_d<128>(tab, sh, Q, K, V, counts_in, alpha_bar, ws, stream, g1, g2, ticks, stagger);
}

}  // namespace kvs
