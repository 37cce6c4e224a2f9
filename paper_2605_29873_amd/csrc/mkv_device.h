// Device-side helpers shared by the attention kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "mkv_internal.h"

namespace mkv {
namespace dev {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// DPP controls: quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror.
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

// Sum over the LPK adjacent lanes that share one key; every lane of the group gets the sum.
template <int LPK>
__device__ __forceinline__ float group_sum(float x) {
  if constexpr (LPK >= 2) x += dpp_mov<kDppXor1>(x);
  if constexpr (LPK >= 4) x += dpp_mov<kDppXor2>(x);
  if constexpr (LPK >= 8) x += dpp_mov<kDppHalfMirror>(x);
  if constexpr (LPK >= 16) x += dpp_mov<kDppMirror>(x);
  return x;
}

// Reductions across the 64/LPK key groups of a wave.  Lane c of every group takes part with lane c
// of the others (row rotations by multiples of LPK, then the two cross-row exchanges), so the same
// code serves values that are uniform inside a group and per-lane accumulators.
constexpr int kDppRowRor = 0x120;
template <int LPK>
__device__ __forceinline__ float across_groups_max(float x) {
  if constexpr (LPK <= 1) x = fmaxf(x, dpp_mov<kDppRowRor + 1>(x));
  if constexpr (LPK <= 2) x = fmaxf(x, dpp_mov<kDppRowRor + 2>(x));
  if constexpr (LPK <= 4) x = fmaxf(x, dpp_mov<kDppRowRor + 4>(x));
  if constexpr (LPK <= 8) x = fmaxf(x, dpp_mov<kDppRowRor + 8>(x));
  x = fmaxf(x, __shfl_xor(x, 16));
  x = fmaxf(x, __shfl_xor(x, 32));
  return x;
}
template <int LPK>
__device__ __forceinline__ float across_groups_sum(float x) {
  if constexpr (LPK <= 1) x += dpp_mov<kDppRowRor + 1>(x);
  if constexpr (LPK <= 2) x += dpp_mov<kDppRowRor + 2>(x);
  if constexpr (LPK <= 4) x += dpp_mov<kDppRowRor + 4>(x);
  if constexpr (LPK <= 8) x += dpp_mov<kDppRowRor + 8>(x);
  x += __shfl_xor(x, 16);
  x += __shfl_xor(x, 32);
  return x;
}

// Values that are equal in every lane of a wave but that the compiler cannot know to be (read
// from LDS or through a lane-indexed path): moving them to scalar registers keeps the address and
// loop arithmetic derived from them off the vector ALU.
// Brings every 64-byte line of the kernel's argument block (BYTES long, at most 1 KiB) into the
// scalar cache with independent loads and one wait.  The compiler fetches arguments where they are
// first used, in several batches that each wait for memory; with a large argument block the batches
// touch one new line after the other and their round trips add up in front of the first key load.
// After this call they hit the cache.
// Written as two blocks of eight scalar loads with the wait at the end of the second: left to the
// compiler the loads come in two batches with a wait after each.  The first block's registers are
// operands of the second, so nothing else is allocated to them while their loads are in flight.
template <int BYTES>
__device__ __forceinline__ void warm_kernel_arguments() {
  static_assert(BYTES >= 64 && BYTES <= 1024, "argument block of one to sixteen lines");
  // line i is touched through its first word, which lies inside the block
#define MKV_LINE(i) ((i) * 64 + 4 <= BYTES ? (i) * 64 : 0)
  const uint64_t base = (uint64_t)__builtin_amdgcn_kernarg_segment_ptr();
  uint32_t t0, t1, t2, t3, t4, t5, t6, t7;
  asm volatile(
      "s_load_dword %0, %8, %9\n\t"
      "s_load_dword %1, %8, %10\n\t"
      "s_load_dword %2, %8, %11\n\t"
      "s_load_dword %3, %8, %12\n\t"
      "s_load_dword %4, %8, %13\n\t"
      "s_load_dword %5, %8, %14\n\t"
      "s_load_dword %6, %8, %15\n\t"
      "s_load_dword %7, %8, %16"
      : "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3), "=&s"(t4), "=&s"(t5), "=&s"(t6), "=&s"(t7)
      : "s"(base), "i"(MKV_LINE(0)), "i"(MKV_LINE(1)), "i"(MKV_LINE(2)), "i"(MKV_LINE(3)), "i"(MKV_LINE(4)),
        "i"(MKV_LINE(5)), "i"(MKV_LINE(6)), "i"(MKV_LINE(7)));
  uint32_t u0, u1, u2, u3, u4, u5, u6, u7;
  asm volatile(
      "s_load_dword %0, %16, %17\n\t"
      "s_load_dword %1, %16, %18\n\t"
      "s_load_dword %2, %16, %19\n\t"
      "s_load_dword %3, %16, %20\n\t"
      "s_load_dword %4, %16, %21\n\t"
      "s_load_dword %5, %16, %22\n\t"
      "s_load_dword %6, %16, %23\n\t"
      "s_load_dword %7, %16, %24\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(u0), "=&s"(u1), "=&s"(u2), "=&s"(u3), "=&s"(u4), "=&s"(u5), "=&s"(u6), "=&s"(u7), "+s"(t0), "+s"(t1),
        "+s"(t2), "+s"(t3), "+s"(t4), "+s"(t5), "+s"(t6), "+s"(t7)
      : "s"(base), "i"(MKV_LINE(8)), "i"(MKV_LINE(9)), "i"(MKV_LINE(10)), "i"(MKV_LINE(11)), "i"(MKV_LINE(12)),
        "i"(MKV_LINE(13)), "i"(MKV_LINE(14)), "i"(MKV_LINE(15)));
#undef MKV_LINE
}

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ long long uniform(long long x) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((int)(uint32_t)x);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((int)(uint32_t)((unsigned long long)x >> 32));
  return (long long)(((unsigned long long)hi << 32) | lo);
}

__device__ __forceinline__ uint4 ldg16(const char* p) { return *reinterpret_cast<const uint4*>(p); }
// Same load with the non-temporal hint: for rows read once per launch by one wave, a whole row per
// lane group, so that nothing is gained from keeping the line in a cache.
__device__ __forceinline__ uint4 ldg16_stream(const char* p) {
  typedef __attribute__((ext_vector_type(4))) unsigned int u4;
  const u4 v = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Prefix sums of the per-sequence key counts, built by one wave into LDS: offs[b] = number of keys
// of all units of sequences < b, where a sequence has `units` = Hkv * passes units of
// L_b = M_b + n_d + n_new positions each (0 for inactive sequences; n_new = tokens appended by the
// step plus the unit's virtual positions).  offs has B+1 entries.  With `il` valid the lengths come with the launch arguments.
__device__ __forceinline__ void build_offsets(const Shape& s, const LayerView& lv, const SeqMask& mask,
                                              int units, int n_new, long long* offs, int lane,
                                              const InlineLens* il = nullptr) {
  if (il && il->valid) {   // at most 32 sequences, prefix sums made by the host
    if (lane <= s.B) offs[lane] = il->offs[lane & (kInlineLens * 2 - 1)];
    return;
  }
  const int per = (s.B + 63) / 64;
  const int b0 = lane * per;
  long long sum = 0;
  for (int i = 0; i < per; ++i) {
    const int b = b0 + i;
    if (b < s.B && mask.active(b)) sum += (long long)units * (lv.mlen[b] + lv.nd[b] + n_new);
  }
  long long incl = sum;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const long long y = __shfl_up(incl, off);
    if (lane >= off) incl += y;
  }
  long long run = incl - sum;
  for (int i = 0; i < per; ++i) {
    const int b = b0 + i;
    if (b < s.B) {
      offs[b] = run;
      if (mask.active(b)) run += (long long)units * (lv.mlen[b] + lv.nd[b] + n_new);
    }
  }
  if (lane == 63) offs[s.B] = incl;
}

// floor(a / b) for 0 <= a < 2^22 and b >= 1 through the float reciprocal and one correction step
// (the integer division is a subroutine of some forty instructions, this is ten).
__device__ __forceinline__ int div_small(int a, int b) {
  int q = (int)((float)a * __frcp_rn((float)b));      // off by one at most
  const int r = a - q * b;
  q += (r >= b) - (r < 0);
  return q;
}

// quad_perm controls that exchange lane i with lane i^K inside every group of four lanes
template <int K>
__device__ __forceinline__ float quad_xor(float x) {
  if constexpr (K == 1) return dpp_mov<0xB1>(x);       // [1,0,3,2]
  else if constexpr (K == 2) return dpp_mov<0x4E>(x);  // [2,3,0,1]
  else if constexpr (K == 3) return dpp_mov<0x1B>(x);  // [3,2,1,0]
  else return x;
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

// Softmax normaliser of one head from its per-piece (reference, sum) pairs, by one whole wave:
// returns the common reference mx and the total sum L relative to it (both base 2).  `ml` points
// at the head's pair in the first slot; consecutive slots are `stride` floats apart.
__device__ __forceinline__ void wave_merge_ml(const float* ml, int stride, int ns, int lane, float& mx, float& L,
                                              float* m_first = nullptr) {
  // the first 64 pieces (nearly always all of them) are held in registers: one round of loads
  const float2 v = lane < ns ? *reinterpret_cast<const float2*>(ml + (size_t)lane * stride)
                             : make_float2(-INFINITY, 0.f);
  float m_loc = v.x;
  for (int i = lane + 64; i < ns; i += 64) m_loc = fmaxf(m_loc, ml[(size_t)i * stride]);
  mx = wave_max(m_loc);
  float l_loc = (v.x == -INFINITY) ? 0.f : fast_exp2(v.x - mx) * v.y;
  for (int i = lane + 64; i < ns; i += 64)
    l_loc = fmaf(fast_exp2(ml[(size_t)i * stride] - mx), ml[(size_t)i * stride + 1], l_loc);
  L = wave_sum(l_loc);
  if (m_first) *m_first = v.x;
}

// Order-preserving map float -> uint32 (total order of the reals; -0 is folded onto +0 so that the
// two zeros tie, as they do under float comparison).
__device__ __forceinline__ uint32_t ordered_key(uint32_t bits) {
  if (bits == 0x80000000u) bits = 0u;
  return (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
}

// Selection key of a slot for Eq. 8: lowest score first, the older slot on a tie.
__device__ __forceinline__ unsigned long long evict_key_of(float score, int slot) {
  return ((unsigned long long)ordered_key(__builtin_bit_cast(uint32_t, score)) << 32) | (uint32_t)slot;
}

// Minimum of `key` over a 256-thread work-group, merged into *dst with one atomic (~0 = no
// candidate): atomics of many waves on one address queue up behind each other.  Every thread of the
// work-group must call it; `slots` is LDS for four values.
__device__ __forceinline__ void block_min_key_to(unsigned long long key, unsigned long long* dst,
                                                 unsigned long long* slots, int tid) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long o = __shfl_xor(key, off);
    key = o < key ? o : key;
  }
  __syncthreads();                      // slots may still be read from the previous call
  if ((tid & 63) == 0) slots[tid >> 6] = key;
  __syncthreads();
  if (tid == 0) {
    unsigned long long m = slots[0];
#pragma unroll
    for (int w = 1; w < 4; ++w) m = slots[w] < m ? slots[w] : m;
    if (m != ~0ull) atomicMin(dst, m);
  }
}

}  // namespace dev
}  // namespace mkv
