// Pieces shared by the bf16 matrix-core score kernels: the 32-token tile, LDS operand reads with explicit waits,
// and the per-tile adjustments of the logits (cardinalities, causal window).
#pragma once

#include "kvs_device.h"

namespace kvs {
namespace mfma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTile = 32;                 // tokens per MFMA tile
constexpr int kNonTemporal = 2;           // cache-policy bit of K tile loads that no later sweep finds cached anyway

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

// Four 16-byte LDS reads at byte addresses ad[0..3] + OFF, complete on return.  Written as inline
// assembly on purpose: the compiler treats every LDS read as dependent on ALL outstanding
// global->LDS loads and would wait for the tile that is still being prefetched into the other buffer;
// here the wait on the right tile is the explicit vmcnt above the call.
template <int OFF>
__device__ __forceinline__ void lds_read_4x16(bf16x8& a0, bf16x8& a1, bf16x8& a2, bf16x8& a3, const uint32_t* ad) {
  asm volatile(
      "ds_read_b128 %0, %4 offset:%8\n\t"
      "ds_read_b128 %1, %5 offset:%8\n\t"
      "ds_read_b128 %2, %6 offset:%8\n\t"
      "ds_read_b128 %3, %7 offset:%8\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(a0), "=&v"(a1), "=&v"(a2), "=&v"(a3)
      : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "n"(OFF)
      : "memory");
}

// Rows that stand for c tokens with one Key (an already merged cache) enter the softmax as c equal
// terms, i.e. with log2(c) added to the base-2 logit.  Turns the raw dot products of this lane's 16
// accumulator rows (tile at token base_t of the unit whose cardinalities start at cnt) into logits.
template <int NACC>
__device__ __forceinline__ void logits_with_counts(f32x16 (&acc)[NACC], const int32_t* __restrict__ cnt, int base_t,
                                                   int half, float sl2) {
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = 8 * (v / 4) + 4 * half + (v % 4);
    const float lc = log2f((float)cnt[base_t + row]);
#pragma unroll
    for (int nt = 0; nt < NACC; ++nt) acc[nt][v] = fmaf(acc[nt][v], sl2, lc);
  }
}

// Causal window: accumulator rows past the last row a query column attends to leave the softmax
// (lim[i]: that row for the query column of accumulator i).
template <int NACC>
__device__ __forceinline__ void mask_causal(f32x16 (&acc)[NACC], const int (&lim)[NACC], int base_t, int half) {
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int t = base_t + 8 * (v / 4) + 4 * half + (v % 4);
#pragma unroll
    for (int i = 0; i < NACC; ++i) {
      if (t > lim[i]) acc[i][v] = -INFINITY;
    }
  }
}

#define KVS_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define KVS_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// Two 16-byte LDS reads at each of two addresses (offsets OFF0 and OFF1), complete on return.
template <int OFF0, int OFF1>
__device__ __forceinline__ void lds_read_2x2(bf16x8& b00, bf16x8& b01, bf16x8& b10, bf16x8& b11, uint32_t ad0,
                                             uint32_t ad1) {
  asm volatile(
      "ds_read_b128 %0, %4 offset:%6\n\t"
      "ds_read_b128 %1, %4 offset:%7\n\t"
      "ds_read_b128 %2, %5 offset:%6\n\t"
      "ds_read_b128 %3, %5 offset:%7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(b00), "=&v"(b01), "=&v"(b10), "=&v"(b11)
      : "v"(ad0), "v"(ad1), "n"(OFF0), "n"(OFF1)
      : "memory");
}

// One 16-byte LDS read at each of two addresses (offset OFF), complete on return.
template <int OFF>
__device__ __forceinline__ void lds_read_2x1(bf16x8& b0, bf16x8& b1, uint32_t ad0, uint32_t ad1) {
  asm volatile(
      "ds_read_b128 %0, %2 offset:%4\n\t"
      "ds_read_b128 %1, %3 offset:%4\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(b0), "=&v"(b1)
      : "v"(ad0), "v"(ad1), "n"(OFF)
      : "memory");
}

}  // namespace mfma
}  // namespace kvs
