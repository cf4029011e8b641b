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
// A slot of one token is copied bit for bit.  Ablation rules (kvs_key_rule): C_t := 0, or u_t := the
// number of tokens row t stands for (arithmetic mean).
//
// COUNTS: the rows are slots of an already merged cache, row t standing for c_t tokens whose Values add
// up to V[t] (Sec. 3.1, streaming regime): r_t = V[t] / c_t - o_bar, counts[S] = sum c_t, the fallback is
// the mean over the tokens the rows stand for; everything else is unchanged.
//
// NORMS: A_t and C_t are not formed from alpha_bar and o_bar but read from two arrays (per-query
// aggregation: every query row with its own attention and output, the norms averaged over the rows);
// the weight form, the Values and the cardinalities are the same.
//
// Work split.  A workgroup is responsible for the slots that BEGIN in its nominal range of
// kMergeTokens tokens: its real range [A, B) runs from the first slot start at or after the
// nominal begin to the first slot start at or after the nominal end, so it owns whole slots and
// never talks to another workgroup.  [A, B) is cut evenly over the workgroup's lane groups (a
// lane group = the LPR adjacent lanes that read one row, 16 bytes each).  A group walks its
// tokens in order with the open slot's accumulators in registers; slots that lie inside the group
// are written directly, the pieces of a slot that crosses group borders (head / through / tail
// fragments) go to LDS and are added up, in group order, by the group in which the slot begins.
// Long runs are therefore summed by many groups in parallel and the result depends only on the
// edge mask and the launch geometry, never on timing (no atomics).
// Rows are requested kPrefetch tokens ahead of their use.
#include "kvs_device.h"

namespace kvs {
namespace {

constexpr int kThreads = 256;
#ifndef KVS_MERGE_PREFETCH
#define KVS_MERGE_PREFETCH 3
#endif
constexpr int kPrefetch = KVS_MERGE_PREFETCH;

template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  return row_group_sum<LPR>(x);
}

// First token t >= from that starts a slot (t == 0 or mask[t-1] == 0); n if there is none.
// Called by the whole workgroup; sm is 1 + kThreads / kWave ints of scratch.
__device__ __forceinline__ int first_slot_start(const uint8_t* __restrict__ mk, int from, int n, int* sm) {
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  for (int base = from;; base += kThreads) {
    const int t = base + tid;
    const bool start = (t >= n) || (t == 0) || (mk[t - 1] == 0);
    const uint64_t bal = __ballot(start);
    if (lane == 0) sm[wave] = bal ? base + wave * kWave + (__ffsll((long long)bal) - 1) : 0x7fffffff;
    __syncthreads();
    int best = 0x7fffffff;
#pragma unroll
    for (int w = 0; w < kThreads / kWave; ++w) best = min(best, sm[w]);
    __syncthreads();
    if (best != 0x7fffffff) return min(best, n);
  }
}

// NORMS: `alpha_bar` holds A_t and `c_edge` C_t (o_bar and o_part are not used); otherwise c_edge is not used.
template <typename T, int D, bool STREAM, bool COUNTS, bool NORMS>
__global__ __launch_bounds__(kThreads) void merge_kernel(
    const UnitTable tab, const Shape sh, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ counts_in, const float* __restrict__ alpha_bar, const float* __restrict__ o_bar, const float* __restrict__ o_part,
    const float* __restrict__ c_edge,
    const uint8_t* __restrict__ edge_mask, const int32_t* __restrict__ slot, T* __restrict__ K_out,
    T* __restrict__ V_out, int32_t* __restrict__ counts) {
  constexpr int EPL = Piece<T>::N;
  constexpr int LPR = D / EPL;
  constexpr int GROUPS = kThreads / LPR;
  constexpr int FRAG = 2 * D + 4;           // accK[D], accV[D], U, rows, first token, cardinality

  __shared__ float sm_frag[GROUPS][2][FRAG];   // [g][0]: head fragment, [g][1]: tail / through fragment
  __shared__ int sm_flag[GROUPS];              // bit 0: head fragment ends here, 1: through, 2: tail starts here
  __shared__ int sm_tail_slot[GROUPS];
  __shared__ int sm_scan[2 * (kThreads / kWave)];
  __shared__ float sm_obar[kThreads / D][D];

  const int ui = find_unit_by<&Unit::m_base>(tab, (int)blockIdx.x);
  const Unit un = tab.unit(ui);
  const int n = un.len;
  const int tid = threadIdx.x;
  const int group = tid / LPR, piece = tid % LPR;
  const uint8_t* mk = edge_mask + un.in_row;

  const int nom_a = ((int)blockIdx.x - un.m_base) * kMergeTokens;
  const int nom_b = min(n, nom_a + kMergeTokens);

  // Everything the prologue needs is requested at once (one round trip): the edge-mask bytes that
  // decide where the workgroup's real range begins and ends, and the chunk sums of o_bar.
  const int wave = tid / kWave, lane = tid % kWave;
  const int ta = nom_a + tid, tb = nom_b + tid;
  const bool start_a = (ta >= n) || (ta == 0) || (mk[ta - 1] == 0);
  const bool start_b = (tb >= n) || (tb == 0) || (mk[tb - 1] == 0);
  constexpr int PARTS = kThreads / D;          // threads per channel when adding up the chunk sums
  constexpr int PER = kMaxChunks / PARTS;
  float part_sum = 0.f;
  if (!NORMS && o_bar == nullptr) {
    const int nc = obar_partials(sh, un);
    const int d = tid % D, h = tid / D;
    float v[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = h * PER + i;
      v[i] = (c < nc) ? o_part[((size_t)un.index * kMaxChunks + c) * D + d] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) part_sum += v[i];
    sm_obar[h][d] = part_sum;
  }
  {
    const uint64_t ba = __ballot(start_a), bb = __ballot(start_b);
    if (lane == 0) {
      sm_scan[wave] = ba ? nom_a + wave * kWave + (__ffsll((long long)ba) - 1) : 0x7fffffff;
      sm_scan[4 + wave] = bb ? nom_b + wave * kWave + (__ffsll((long long)bb) - 1) : 0x7fffffff;
    }
  }
  __syncthreads();
  int A = 0x7fffffff, B = 0x7fffffff;
#pragma unroll
  for (int w = 0; w < kThreads / kWave; ++w) { A = min(A, sm_scan[w]); B = min(B, sm_scan[4 + w]); }
  __syncthreads();
  // a slot longer than the probe window: keep looking (rare)
  A = (A == 0x7fffffff) ? first_slot_start(mk, nom_a + kThreads, n, sm_scan) : min(A, n);
  B = (B == 0x7fffffff) ? first_slot_start(mk, nom_b + kThreads, n, sm_scan) : min(B, n);
  if (A >= B) return;                          // the whole nominal range lies inside a slot owned earlier

  // Unit-wide base pointers (uniform: they live in scalar registers) plus 32-bit byte offsets per lane:
  // a unit's rows span less than 4 GB (the host checks the length), and a 32-bit offset costs one
  // instruction per address where a 64-bit per-lane pointer costs four.
  constexpr uint32_t ROWB = D * sizeof(T);
  const char* Kb = reinterpret_cast<const char*>(K + (size_t)un.in_row * D);
  const char* Vb = reinterpret_cast<const char*>(V + (size_t)un.in_row * D);
  char* Kob = reinterpret_cast<char*>(K_out + (size_t)un.out_row * D);
  char* Vob = reinterpret_cast<char*>(V_out + (size_t)un.out_row * D);
  const uint32_t pofs = piece * 16;
  // When the launch's rows exceed the caches they are read once and written once as far as any cache
  // is concerned: non-temporal accesses then keep them from displacing one another in L2 (measured:
  // about 3 % each for the loads and the stores).  Smaller launches find K and V where the sweeps
  // before left them and keep the ordinary policy.
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  auto load_row = [&](const char* base, int t) {
    const u32x4* src = reinterpret_cast<const u32x4*>(base + ((uint32_t)t * ROWB + pofs));
    const u32x4 r = STREAM ? __builtin_nontemporal_load(src) : *src;
    return make_uint4(r.x, r.y, r.z, r.w);
  };
  auto store_row = [&](char* base, int t, const uint4& x) {
    const u32x4 r = {x.x, x.y, x.z, x.w};
    u32x4* dst = reinterpret_cast<u32x4*>(base + ((uint32_t)t * ROWB + pofs));
    if (STREAM) __builtin_nontemporal_store(r, dst);
    else *dst = r;
  };
  auto k_row = [&](int t) { return load_row(Kb, t); };
  auto v_row = [&](int t) { return load_row(Vb, t); };
  int32_t* cnt = counts + un.out_row;
  const float* al = alpha_bar + un.in_row;
  const float* ce = NORMS ? c_edge + un.in_row : nullptr;
  auto cedge_at = [&](int t) { return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(ce) + (uint32_t)t * 4u); };
  const int32_t* sl = slot + un.in_row;
  auto alpha_at = [&](int t) { return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(al) + (uint32_t)t * 4u); };
  auto mask_at = [&](int t) { return *(mk + (uint32_t)t); };
  const int32_t* cin = COUNTS ? counts_in + un.in_row : nullptr;
  auto count_at = [&](int t) { return COUNTS ? *reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(cin) + (uint32_t)t * 4u) : 1; };

  // o_bar: final values, or the chunk sums added in a fixed order (every workgroup gets the same bits)
  float o[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int d = piece * EPL + i;
    if (NORMS) {
      o[i] = 0.f;
    } else if (o_bar != nullptr) {
      o[i] = o_bar[(size_t)un.index * D + d];
    } else {
      float s = sm_obar[0][d];
#pragma unroll
      for (int h = 1; h < PARTS; ++h) s += sm_obar[h][d];
      o[i] = s;
    }
  }

  // One finished slot -> global memory (all lanes of the group call it together).  `raw_*` are the
  auto finish = [&](int out_slot, const float* accK, const float* accV, float U, int count, int csum, int first_tok,
                    const uint4& raw_k) {
    float outk[EPL];
    if (U > 0.f && U < INFINITY) {
      const float inv = __builtin_amdgcn_rcpf(U);
#pragma unroll
      for (int i = 0; i < EPL; ++i) outk[i] = accK[i] * inv;
    } else {                                   // no usable weights: arithmetic mean of the run
#pragma unroll
      for (int i = 0; i < EPL; ++i) outk[i] = 0.f;
      for (int j = first_tok; j < first_tok + count; ++j) {
        float kj[EPL];
        Piece<T>::unpack(k_row(j), kj);
        const float cj = (float)count_at(j);
#pragma unroll
        for (int i = 0; i < EPL; ++i) outk[i] = fmaf(cj, kj[i], outk[i]);
      }
      const float inv = 1.f / (float)csum;
#pragma unroll
      for (int i = 0; i < EPL; ++i) outk[i] *= inv;
    }
    uint4 ok = Piece<T>::pack(outk);
    const uint4 ov = Piece<T>::pack(accV);       // a single row converts back to its own bits
    if (count == 1) ok = raw_k;
    if ((unsigned)out_slot < (unsigned)un.n_out) {   // a slot map from outside the library is not trusted
      store_row(Kob, out_slot, ok);
      store_row(Vob, out_slot, ov);
      if (piece == 0) *reinterpret_cast<int32_t*>(reinterpret_cast<char*>(cnt) + (uint32_t)out_slot * 4u) = csum;
    }
  };
  auto store_frag = [&](float* f, const float* accK, const float* accV, float U, int count, int csum, int first_tok) {
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      f[piece * EPL + i] = accK[i];
      f[D + piece * EPL + i] = accV[i];
    }
    if (piece == 0) {
      f[2 * D] = U;
      f[2 * D + 1] = __int_as_float(count);
      f[2 * D + 2] = __int_as_float(first_tok);
      f[2 * D + 3] = __int_as_float(csum);
    }
  };

  // ablations of the Key rule (uniform): no coupling blocks, or plain token-count weights
  const bool coupled = sh.rule == KVS_RULE_HESSIAN;
  const bool mean_rule = sh.rule == KVS_RULE_MEAN;
  const int per = (B - A + GROUPS - 1) / GROUPS;
  const int ga = A + group * per;
  const int gb = min(B, ga + per);
  int flags = 0, tail_slot = 0;

  if (ga < gb) {
    const bool head_open = (ga > A) && (mk[ga - 1] != 0);
    // Token t's weight needs C_t, i.e. the NEXT token's Value row: the walk therefore reads V one token
    // ahead of K, and the last step looks at row gb (which exists whenever the slot is still open).
    const int last_v = min(gb, n - 1);
    const int out_slot0 = sl[ga];                    // slots are numbered consecutively from here

    // kPrefetch register sets (K row, the Value row one token later, its alpha and edge bit), used in
    // rotation by an equally unrolled loop: a set is refilled for token t + kPrefetch at the end of
    // the step that consumed it, so no set is ever copied and a step waits for its own set only.
    uint4 rk[kPrefetch], rv[kPrefetch];
    float ra[kPrefetch];
    uint8_t rm[kPrefetch];          // kept as loaded: widening at the load would wait for it there
    int rc[kPrefetch];              // cardinality of the Value row's token (COUNTS only)
    float re[kPrefetch];            // C of the edge after the Value row's token (NORMS only)
    auto refill = [&](int j, int t) {                // the set that token t will consume
      rk[j] = k_row(min(t, gb - 1));
      const int tv = min(t + 1, last_v);
      rv[j] = v_row(tv);
      ra[j] = alpha_at(tv);
      rm[j] = mask_at(tv);
      if (COUNTS) rc[j] = count_at(tv);
      if (NORMS) re[j] = cedge_at(tv);
    };
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) refill(j, ga + j);
    const uint4 vraw_first = v_row(ga);
    float alpha_cur = al[ga];
    uint32_t mask_cur = mk[ga];

    float v_cur[EPL], r_cur[EPL], accK[EPL], accV[EPL];
    float ss_cur = 0.f, Cprev = 0.f, U = 0.f;
    float ce_cur = NORMS ? ce[ga] : 0.f;             // NORMS: C of the edge after the current token
    int count = 0, first_tok = ga, out_slot = out_slot0;
    int c_cur = count_at(ga), csum = 0;              // COUNTS: this row's cardinality, the open slot's so far
    bool is_head = head_open;       // the open slot began before this group
    if (NORMS) {
      Piece<T>::unpack(vraw_first, v_cur);
#pragma unroll
      for (int i = 0; i < EPL; ++i) { r_cur[i] = 0.f; accK[i] = 0.f; accV[i] = 0.f; }
      Cprev = (head_open && coupled) ? ce[ga - 1] : 0.f;
    } else {
      Piece<T>::unpack(vraw_first, v_cur);
      const float ic0 = COUNTS ? __builtin_amdgcn_rcpf((float)c_cur) : 1.f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        r_cur[i] = COUNTS ? fmaf(v_cur[i], ic0, -o[i]) : v_cur[i] - o[i];
        ss_cur = fmaf(r_cur[i], r_cur[i], ss_cur);
        accK[i] = 0.f;
        accV[i] = 0.f;
      }
      float dot = 0.f, ss_b = 0.f;
      float a_before = 0.f;
      if (head_open) {                               // C_{ga-1} from the row before the group
        float vb[EPL];
        Piece<T>::unpack(v_row(ga - 1), vb);
        a_before = al[ga - 1];
        const float icb = COUNTS ? __builtin_amdgcn_rcpf((float)count_at(ga - 1)) : 1.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
          const float rb = COUNTS ? fmaf(vb[i], icb, -o[i]) : vb[i] - o[i];
          ss_b = fmaf(rb, rb, ss_b);
          dot = fmaf(rb, r_cur[i], dot);
        }
      }
      ss_cur = group_sum<LPR>(ss_cur);
      ss_b = group_sum<LPR>(ss_b);
      dot = group_sum<LPR>(dot);
      Cprev = coupled ? a_before * alpha_cur * __builtin_amdgcn_sqrtf(fmaxf(fmaf(2.f, dot, ss_b + ss_cur), 0.f)) : 0.f;
    }

    // One token.  The same straight-line code for every token: lane groups of a wavefront stay converged.
    auto step = [&](int t, int j) {
      const uint4 kraw = rk[j], vraw_n = rv[j];
      // alpha and the edge bit outlive this step (they are the next step's current token): move them
      // out of the set here, or the refill below is given other registers and copied back after a wait
      float alpha_n;
      uint32_t mask_n;
      asm volatile("v_mov_b32 %0, %2\n\tv_mov_b32 %1, %3"
                   : "=&v"(alpha_n), "=&v"(mask_n)
                   : "v"(ra[j]), "v"((uint32_t)rm[j]));
      int c_n = 1;
      if (COUNTS) asm volatile("v_mov_b32 %0, %1" : "=&v"(c_n) : "v"(rc[j]));
      float ce_n = 0.f;
      if (NORMS) asm volatile("v_mov_b32 %0, %1" : "=&v"(ce_n) : "v"(re[j]));
      const float icn = COUNTS ? __builtin_amdgcn_rcpf((float)c_n) : 1.f;
      // the unit's last token has no edge after it, whatever its mask byte says (an edge mask that comes from
      // outside the library is not trusted to keep that byte at zero)
      const uint32_t edge = (t == n - 1) ? 0u : mask_cur;
      float kf[EPL], vn[EPL], r_next[EPL];
      Piece<T>::unpack(kraw, kf);
      Piece<T>::unpack(vraw_n, vn);
      // ||r_t + r_{t+1}||^2 = ||r_t||^2 + ||r_{t+1}||^2 + 2 r_t . r_{t+1}
      float ss_next = 0.f, dot = 0.f;
      float Anorm, C;
      if (NORMS) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) r_next[i] = 0.f;
        Anorm = alpha_cur;
        C = (edge && coupled) ? ce_cur : 0.f;
      } else {
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
          r_next[i] = COUNTS ? fmaf(vn[i], icn, -o[i]) : vn[i] - o[i];
          ss_next = fmaf(r_next[i], r_next[i], ss_next);
          dot = fmaf(r_cur[i], r_next[i], dot);
        }
        ss_next = group_sum<LPR>(ss_next);
        dot = group_sum<LPR>(dot);
        Anorm = alpha_cur * fabsf(1.f - 2.f * alpha_cur) * __builtin_amdgcn_sqrtf(ss_cur);
        const float pair2 = fmaxf(fmaf(2.f, dot, ss_cur + ss_next), 0.f);
        C = (edge && coupled) ? alpha_cur * alpha_n * __builtin_amdgcn_sqrtf(pair2) : 0.f;
      }
      const float u = mean_rule ? (float)c_cur : Anorm - Cprev - C;
      first_tok = (count == 0) ? t : first_tok;
      U += u;
      ++count;
      if (COUNTS) csum += c_cur;
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        accK[i] = fmaf(u, kf[i], accK[i]);
        accV[i] += v_cur[i];
      }
      if (edge == 0) {                               // the slot ends at t
        if (is_head) {
          store_frag(sm_frag[group][0], accK, accV, U, count, COUNTS ? csum : count, first_tok);
          flags |= 1;
          is_head = false;
        } else {
          finish(out_slot, accK, accV, U, count, COUNTS ? csum : count, first_tok, kraw);
        }
        ++out_slot;
        U = 0.f;
        count = 0;
        csum = 0;
#pragma unroll
        for (int i = 0; i < EPL; ++i) { accK[i] = 0.f; accV[i] = 0.f; }
      }
      refill(j, t + kPrefetch);
      c_cur = c_n;
      ce_cur = ce_n;
      Cprev = C;
      ss_cur = ss_next;
      alpha_cur = alpha_n;
      mask_cur = mask_n;
#pragma unroll
      for (int i = 0; i < EPL; ++i) { r_cur[i] = r_next[i]; v_cur[i] = vn[i]; }
    };

    int t = ga;
    for (; t + kPrefetch <= gb; t += kPrefetch) {
#pragma unroll
      for (int j = 0; j < kPrefetch; ++j) step(t + j, j);
    }
#pragma unroll
    for (int j = 0; j < kPrefetch - 1; ++j) {
      if (t + j < gb) step(t + j, j);
    }
    if (count > 0) {                                 // a slot is still open at the end of the group
      store_frag(sm_frag[group][1], accK, accV, U, count, COUNTS ? csum : count, first_tok);
      if (is_head) {
        flags |= 2;                                  // the whole group lies inside one slot
      } else {
        flags |= 4;                                  // the slot began in this group
        tail_slot = out_slot;
      }
    }
  }
  if (piece == 0) { sm_flag[group] = flags; sm_tail_slot[group] = tail_slot; }
  __syncthreads();

  if (flags & 4) {
    // this group owns a slot that continues in later groups: add their fragments in group order
    float accK[EPL], accV[EPL];
    const float* f = sm_frag[group][1];
#pragma unroll
    for (int i = 0; i < EPL; ++i) { accK[i] = f[piece * EPL + i]; accV[i] = f[D + piece * EPL + i]; }
    float U = f[2 * D];
    int count = __float_as_int(f[2 * D + 1]);
    const int first_tok = __float_as_int(f[2 * D + 2]);
    int csum = __float_as_int(f[2 * D + 3]);
    for (int g = group + 1; g < GROUPS; ++g) {
      const int fl = sm_flag[g];
      const float* h = sm_frag[g][(fl & 2) ? 1 : 0];
      if (!(fl & 3)) break;                        // cannot happen for a consistent mask
#pragma unroll
      for (int i = 0; i < EPL; ++i) { accK[i] += h[piece * EPL + i]; accV[i] += h[D + piece * EPL + i]; }
      U += h[2 * D];
      count += __float_as_int(h[2 * D + 1]);
      csum += __float_as_int(h[2 * D + 3]);
      if (fl & 1) break;                           // the slot ended in group g
    }
    finish(tail_slot, accK, accV, U, count, csum, first_tok, make_uint4(0, 0, 0, 0));
  }
}

}  // namespace

template <typename T, int D, bool STREAM, bool COUNTS, bool NORMS = false>
static hipError_t launch_merge_k(const UnitTable& tab, const Shape& sh, const void* K, const void* V,
                                 const int32_t* counts_in, const float* alpha_bar, const float* o_bar,
                                 const float* o_part, const uint8_t* edge_mask, const int32_t* slot, void* K_out,
                                 void* V_out, int32_t* counts, hipStream_t stream, const float* c_edge = nullptr) {
  hipLaunchKernelGGL((merge_kernel<T, D, STREAM, COUNTS, NORMS>), dim3(tab.total_mblocks), dim3(kThreads), 0, stream,
                     tab, sh, (const T*)K, (const T*)V, counts_in, alpha_bar, o_bar, o_part, c_edge, edge_mask, slot,
                     (T*)K_out, (T*)V_out, counts);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_merge_t(const UnitTable& tab, const Shape& sh, const void* K, const void* V,
                                 const int32_t* counts_in, const float* alpha_bar, const float* o_bar,
                                 const float* o_part, const uint8_t* edge_mask, const int32_t* slot, void* K_out,
                                 void* V_out, int32_t* counts, hipStream_t stream) {
#define KVS_MERGE_ARGS tab, sh, K, V, counts_in, alpha_bar, o_bar, o_part, edge_mask, slot, K_out, V_out, counts, stream
  if (counts_in) {
    return sh.stream ? launch_merge_k<T, D, true, true>(KVS_MERGE_ARGS) : launch_merge_k<T, D, false, true>(KVS_MERGE_ARGS);
  }
  return sh.stream ? launch_merge_k<T, D, true, false>(KVS_MERGE_ARGS) : launch_merge_k<T, D, false, false>(KVS_MERGE_ARGS);
}

hipError_t launch_merge(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* K, const void* V,
                        const int32_t* counts_in, const float* alpha_bar, const float* o_bar, const float* o_part,
                        const uint8_t* edge_mask, const int32_t* slot, void* K_out, void* V_out, int32_t* counts,
                        hipStream_t stream) {
  if (dt == KVS_F32) {
    return sh.D == 64 ? launch_merge_t<float, 64>(KVS_MERGE_ARGS) : launch_merge_t<float, 128>(KVS_MERGE_ARGS);
  }
  return sh.D == 64 ? launch_merge_t<uint16_t, 64>(KVS_MERGE_ARGS) : launch_merge_t<uint16_t, 128>(KVS_MERGE_ARGS);
#undef KVS_MERGE_ARGS
}

template <typename T, int D>
static hipError_t launch_merge_norms_t(const UnitTable& tab, const Shape& sh, const void* K, const void* V,
                                       const int32_t* counts_in, const float* a_tok, const float* c_edge,
                                       const uint8_t* edge_mask, const int32_t* slot, void* K_out, void* V_out,
                                       int32_t* counts, hipStream_t stream) {
#define KVS_MN_ARGS tab, sh, K, V, counts_in, a_tok, nullptr, nullptr, edge_mask, slot, K_out, V_out, counts, stream, c_edge
  if (counts_in) {
    return sh.stream ? launch_merge_k<T, D, true, true, true>(KVS_MN_ARGS) : launch_merge_k<T, D, false, true, true>(KVS_MN_ARGS);
  }
  return sh.stream ? launch_merge_k<T, D, true, false, true>(KVS_MN_ARGS) : launch_merge_k<T, D, false, false, true>(KVS_MN_ARGS);
#undef KVS_MN_ARGS
}

hipError_t launch_merge_norms(const UnitTable& tab, const Shape& sh, kvs_dtype dt, const void* K, const void* V,
                              const int32_t* counts_in, const float* a_tok, const float* c_edge,
                              const uint8_t* edge_mask, const int32_t* slot, void* K_out, void* V_out, int32_t* counts,
                              hipStream_t stream) {
#define KVS_MN_ARGS tab, sh, K, V, counts_in, a_tok, c_edge, edge_mask, slot, K_out, V_out, counts, stream
  if (dt == KVS_F32) {
    return sh.D == 64 ? launch_merge_norms_t<float, 64>(KVS_MN_ARGS) : launch_merge_norms_t<float, 128>(KVS_MN_ARGS);
  }
  return sh.D == 64 ? launch_merge_norms_t<uint16_t, 64>(KVS_MN_ARGS) : launch_merge_norms_t<uint16_t, 128>(KVS_MN_ARGS);
#undef KVS_MN_ARGS
}

}  // namespace kvs
