// Split-K single-query attention over (prefill pool U decode pool) with logit emission for the
// decode keys, and the finishing kernel that merges the splits, writes Att_t and applies the
// head-mean + momentum update.  Paper: KV-cache preliminaries Eq. 2; Moment-KV Eq. 4-6;
// Algorithm 1 lines "append", "Softmax", "Mean", slice, and the importance loop.
//
// gfx950 only.  One wavefront = 64 lanes.  No matrix cores: per KV byte there are only G
// multiply-adds (G = query heads per KV head), so the kernel is a bandwidth-bound stream over K
// and V with the arithmetic on the vector ALU.
#include "mkv_internal.h"

#include <math.h>

namespace mkv {
namespace {


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

__device__ __forceinline__ uint4 ldg16(const char* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// <k, q> over one 16-byte vector, added to acc.  bf16: two products per v_dot2c_f32_bf16
// (products of bf16 pairs are exact in fp32; the sum is fp32).
template <bool BF16>
__device__ __forceinline__ float dot_vec(const uint4& k, const uint4& q, float acc) {
  if constexpr (BF16) {
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.x), __builtin_bit_cast(bf16x2_t, q.x), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.y), __builtin_bit_cast(bf16x2_t, q.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.z), __builtin_bit_cast(bf16x2_t, q.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.w), __builtin_bit_cast(bf16x2_t, q.w), acc, false);
  } else {
    acc = fmaf(as_f(k.x), as_f(q.x), acc);
    acc = fmaf(as_f(k.y), as_f(q.y), acc);
    acc = fmaf(as_f(k.z), as_f(q.z), acc);
    acc = fmaf(as_f(k.w), as_f(q.w), acc);
  }
  return acc;
}

// acc[0..EPV) += p * v over one 16-byte vector.
template <bool BF16>
__device__ __forceinline__ void axpy_vec(float p, const uint4& v, float* acc) {
  if constexpr (BF16) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      acc[2 * r] = fmaf(p, as_f(w[r] << 16), acc[2 * r]);
      acc[2 * r + 1] = fmaf(p, as_f(w[r] & 0xffff0000u), acc[2 * r + 1]);
    }
  } else {
    acc[0] = fmaf(p, as_f(v.x), acc[0]);
    acc[1] = fmaf(p, as_f(v.y), acc[1]);
    acc[2] = fmaf(p, as_f(v.z), acc[2]);
    acc[3] = fmaf(p, as_f(v.w), acc[3]);
  }
}

struct AttnArgs {
  Shape s;
  LayerView lv;
  Scratch sc;
  const char* q;
  const char* k_new;
  const char* v_new;
  SeqMask mask;
  int passes;  // head passes per KV head: ceil(G / head lanes)
};

// quad_perm controls that exchange lane i with lane i^K inside every group of four lanes
template <int K>
__device__ __forceinline__ float quad_xor(float x) {
  if constexpr (K == 1) return dpp_mov<0xB1>(x);       // [1,0,3,2]
  else if constexpr (K == 2) return dpp_mov<0x4E>(x);  // [2,3,0,1]
  else if constexpr (K == 3) return dpp_mov<0x1B>(x);  // [3,2,1,0]
  else return x;
}

// Work-group (split, kv head x pass, seq): streams keys [j0, jn) of one segment (prefill or
// decode) of one KV head, for up to HL of its query heads, and leaves an un-normalised partial
// (reference, sum, sum p*V) per head.
//
// Lane layout.  LPK adjacent lanes share a key; lane c of a group holds the 16-byte vectors
// c, c+LPK, ... of the row, so one load instruction of a wave reads 64/LPK rows x (LPK*16)
// contiguous bytes.  Inside a key group, lane c is additionally the OWNER of head "hm" = c mod HL:
//   - every lane forms partial dot products for all HL heads, stored relative to its own head
//     (x[k] belongs to head hm^k), so that a log2(HL)-stage reduce-scatter over DPP lane exchanges
//     leaves each lane with the full logit of its own head only: HL-1 + log2(LPK/HL) adds per
//     key instead of HL*log2(LPK);
//   - the softmax (max tracking, exp2, running sum) is done once per (key, head) by the owner
//     lanes instead of LPK times;
//   - for p*V each lane needs the probabilities of all HL heads: they are fetched from the owner
//     lanes with quad_perm DPP reads (plus one half-row mirror when HL = 8).
// With HL = 8 the three exchanges are "xor 7" (row_half_mirror), xor 2 and xor 1, which span the
// eight lanes; head numbers are the lane's coordinates in that basis.
template <bool BF16, int D, int HL, int LPK, int IT, int WPB, bool PF, bool DIAG = false>
__global__ __launch_bounds__(WPB * 64) void attn_split_kernel(const AttnArgs a) {
  constexpr int kWaves = WPB;
  constexpr int kThreads = WPB * 64;
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int ROWB = D * ES;
  constexpr int NV = ROWB / 16;
  constexpr int VPL = NV / LPK;
  constexpr int EPV = 16 / ES;
  constexpr int KPW = 64 / LPK;
  constexpr int TK = KPW * IT;
  static_assert(NV % LPK == 0 && VPL >= 1, "row must split evenly over the lane group");
  static_assert(HL == 1 || HL == 2 || HL == 4 || HL == 8, "head lanes");
  static_assert(LPK % HL == 0 && (LPK == 16 || LPK == 8), "lane group");

  const Shape& s = a.s;
  const int b = blockIdx.z;
  if (!a.mask.active(b)) return;
  const int split = blockIdx.x;
  const int g = blockIdx.y / a.passes;
  const int pass = blockIdx.y - g * a.passes;
  const int M = a.lv.mlen[b];
  const int n0 = a.lv.nd[b];
  const int n1 = n0 + 1;  // the pool the softmax sees includes the token appended now
  const int CH = s.CH;
  const int cp = (M + CH - 1) / CH;
  const int cd = (n1 + CH - 1) / CH;
  if (split >= cp + cd) return;
  const bool dec = split >= cp;
  const int j0 = (dec ? split - cp : split) * CH;
  const int jn = min(dec ? n1 : M, j0 + CH);
  const int jnew = dec ? n0 : -1;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int c = lane % LPK;
  const int kg = lane / LPK;

  // head owned by this lane, as coordinates in the exchange basis (see above)
  int hm;
  if constexpr (HL == 8) {
    const int i = c & 7, hi = i >> 2;
    hm = (hi << 2) | ((((i >> 1) & 1) ^ hi) << 1) | ((i & 1) ^ hi);
  } else {
    hm = c & (HL - 1);
  }

  const size_t head_row = (size_t)b * s.Hkv + g;
  const size_t pool_rows = dec ? (size_t)s.dstride : (size_t)s.pstride;
  const char* kbase = (const char*)(dec ? a.lv.Kd : a.lv.Kp) + head_row * pool_rows * ROWB;
  const char* vbase = (const char*)(dec ? a.lv.Vd : a.lv.Vp) + head_row * pool_rows * ROWB;
  const char* knew = a.k_new + head_row * ROWB;
  const char* vnew = a.v_new + head_row * ROWB;

  if (split == 0 && blockIdx.y == 0 && tid == 0) a.lv.nd_eff[b] = n1;

  // Append (Alg. 1: pool_d <- pool_d U {(K_t, V_t)}): the work-group whose range holds the new
  // slot stores the row for later steps; in this step every reader takes it from k_new / v_new.
  if (dec && pass == 0 && jnew >= j0 && jnew < jn && tid < 2 * NV) {
    const int vsel = tid / NV, vec = tid - vsel * NV;
    const char* src = (vsel ? vnew : knew) + vec * 16;
    char* dst = (char*)(vsel ? a.lv.Vd : a.lv.Kd) + (head_row * pool_rows + (size_t)jnew) * ROWB + vec * 16;
    *reinterpret_cast<uint4*>(dst) = ldg16(src);
  }

  // queries in storage form at this lane's vector positions; qv[k] belongs to head hm ^ k
  uint4 qv[HL][VPL];
#pragma unroll
  for (int k = 0; k < HL; ++k) {
    const int hl = pass * HL + (hm ^ k);
#pragma unroll
    for (int vi = 0; vi < VPL; ++vi) {
      qv[k][vi] = (hl < s.G) ? ldg16(a.q + ((size_t)b * s.H + g * s.G + hl) * ROWB + (vi * LPK + c) * 16)
                             : make_uint4(0, 0, 0, 0);
    }
  }
  const int h_own = pass * HL + hm;                    // head within the KV group
  const bool own_valid = h_own < s.G;
  float* const logit_row = a.sc.logits + ((size_t)b * s.H + g * s.G + (own_valid ? h_own : 0)) * s.cap;
  const bool stash = dec && own_valid && c < HL;       // first owner lane of each head writes

  float m_own = -INFINITY, l_own = 0.f;
  float acc[HL][VPL][EPV];                             // acc[k] belongs to head hm ^ k
#pragma unroll
  for (int k = 0; k < HL; ++k)
#pragma unroll
    for (int vi = 0; vi < VPL; ++vi)
#pragma unroll
      for (int e = 0; e < EPV; ++e) acc[k][vi][e] = 0.f;

  const int ntile = (jn - j0 + TK - 1) / TK;

  auto load_tile = [&](int tt, uint4 (&kr)[IT][VPL], uint4 (&vr)[IT][VPL]) {
    const int jb = j0 + tt * TK;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int j = min(jb + it * KPW + kg, jn - 1);  // clamp: masked later
      const bool isnew = (j == jnew);
      const char* kp = isnew ? knew : kbase + (size_t)j * ROWB;
      const char* vp = isnew ? vnew : vbase + (size_t)j * ROWB;
#pragma unroll
      for (int vi = 0; vi < VPL; ++vi) {
        kr[it][vi] = ldg16(kp + (vi * LPK + c) * 16);
        vr[it][vi] = ldg16(vp + (vi * LPK + c) * 16);
      }
    }
  };

  // One tile: logits of IT keys per lane group, softmax update by the owner lanes, value
  // accumulation.  Each owner lane keeps its own running reference m_own, raised only when a
  // tile's maximum exceeds it by more than kSlack (base-2 units): exp2(s - m) then stays below
  // 2^kSlack, far from overflow, and the rescale is rare.  Lane groups are merged after the loop.
  constexpr float kSlack = 8.0f;
  auto compute_tile = [&](int tt, const uint4 (&kr)[IT][VPL], const uint4 (&vr)[IT][VPL]) {
    if constexpr (DIAG) {  // tuning aid: memory stream only, no attention math (results are garbage)
      uint32_t x = 0;
#pragma unroll
      for (int it = 0; it < IT; ++it)
#pragma unroll
        for (int vi = 0; vi < VPL; ++vi)
          x ^= kr[it][vi].x ^ kr[it][vi].y ^ kr[it][vi].z ^ kr[it][vi].w ^ vr[it][vi].x ^ vr[it][vi].y ^ vr[it][vi].z ^ vr[it][vi].w;
      l_own += as_f(x & 0x3f800000u);
      return;
    }
    const int jb = j0 + tt * TK;
    float sc[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int j = jb + it * KPW + kg;
      float x[HL];
#pragma unroll
      for (int k = 0; k < HL; ++k) {
        float d = 0.f;
#pragma unroll
        for (int vi = 0; vi < VPL; ++vi) d = dot_vec<BF16>(kr[it][vi], qv[k][vi], d);
        x[k] = d;
      }
      // reduce-scatter over the HL lanes that own the heads ...
      if constexpr (HL == 8) {
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] += dpp_mov<kDppHalfMirror>(x[k ^ 4]);
      }
      if constexpr (HL >= 4) {
#pragma unroll
        for (int k = 0; k < 2; ++k) x[k] += quad_xor<2>(x[k ^ 2]);
      }
      if constexpr (HL >= 2) x[0] += quad_xor<1>(x[1]);
      // ... then over the LPK/HL lane sets of the key group (same owner position in each)
      float d = x[0];
      if constexpr (LPK == 16) {
        if constexpr (HL <= 1) d += dpp_mov<kDppRowRor + 1>(d);
        if constexpr (HL <= 2) d += dpp_mov<kDppRowRor + 2>(d);
        if constexpr (HL <= 4) d += dpp_mov<kDppRowRor + 4>(d);
        d += dpp_mov<kDppRowRor + 8>(d);
      } else {  // 8 lanes per key: two keys share a 16-lane row, so rotations would mix keys
        if constexpr (HL <= 1) d += quad_xor<1>(d);
        if constexpr (HL <= 2) d += quad_xor<2>(d);
        if constexpr (HL <= 4) d += __shfl_xor(d, 4);
      }
      d *= s.scale_log2;
      sc[it] = (j < jn) ? d : -INFINITY;
      if (stash && j < jn) logit_row[j] = d;
    }
    float tm = sc[0];
#pragma unroll
    for (int it = 1; it < IT; ++it) tm = fmaxf(tm, sc[it]);
    const bool up = tm > m_own + kSlack;   // also true for the first finite score (m = -inf)
    if (__any(up)) {
      const float mn = up ? tm : m_own;
      const float cf = up ? fast_exp2(m_own - mn) : 1.0f;   // exp2(-inf) = 0 on the first raise
      float cf_o = 0.f;
      if constexpr (HL == 8) cf_o = dpp_mov<kDppHalfMirror>(cf);
      l_own *= cf;
      m_own = mn;
      // per-head factors, fetched from the owner lanes
      float cfs[HL];
      cfs[0] = cf;
      if constexpr (HL >= 2) cfs[1] = quad_xor<1>(cf);
      if constexpr (HL >= 4) { cfs[2] = quad_xor<2>(cf); cfs[3] = quad_xor<3>(cf); }
      if constexpr (HL == 8) {
        cfs[4] = cf_o; cfs[5] = quad_xor<1>(cf_o); cfs[6] = quad_xor<2>(cf_o); cfs[7] = quad_xor<3>(cf_o);
      }
#pragma unroll
      for (int k = 0; k < HL; ++k)
#pragma unroll
        for (int vi = 0; vi < VPL; ++vi)
#pragma unroll
          for (int e = 0; e < EPV; ++e) acc[k][vi][e] *= cfs[k];
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      // a lane set that has seen no key yet has m = -inf and only masked scores: guard exp2(nan)
      const float p = (sc[it] == -INFINITY) ? 0.f : fast_exp2(sc[it] - m_own);
      l_own += p;
      float ps[HL];
      ps[0] = p;
      if constexpr (HL >= 2) ps[1] = quad_xor<1>(p);
      if constexpr (HL >= 4) { ps[2] = quad_xor<2>(p); ps[3] = quad_xor<3>(p); }
      if constexpr (HL == 8) {
        const float po = dpp_mov<kDppHalfMirror>(p);
        ps[4] = po; ps[5] = quad_xor<1>(po); ps[6] = quad_xor<2>(po); ps[7] = quad_xor<3>(po);
      }
#pragma unroll
      for (int k = 0; k < HL; ++k)
#pragma unroll
        for (int vi = 0; vi < VPL; ++vi) axpy_vec<BF16>(ps[k], vr[it][vi], acc[k][vi]);
    }
  };

  if constexpr (PF) {
    // two register buffers, loop unrolled by two so that the prefetch needs no register copies
    uint4 ka[IT][VPL], va[IT][VPL], kb[IT][VPL], vb[IT][VPL];
    if (wave < ntile) load_tile(wave, ka, va);
    for (int tt = wave; tt < ntile; tt += 2 * kWaves) {
      if (tt + kWaves < ntile) load_tile(tt + kWaves, kb, vb);
      compute_tile(tt, ka, va);
      if (tt + kWaves >= ntile) break;
      if (tt + 2 * kWaves < ntile) load_tile(tt + 2 * kWaves, ka, va);
      compute_tile(tt + kWaves, kb, vb);
    }
  } else {
    // no software prefetch: the other waves of the SIMD cover the load latency
    for (int tt = wave; tt < ntile; tt += kWaves) {
      uint4 ka[IT][VPL], va[IT][VPL];
      load_tile(tt, ka, va);
      compute_tile(tt, ka, va);
    }
  }

  // merge the lane sets of the wave: common reference per head, then sums across key groups
  // (and across the LPK/HL owner sets inside a key group for the running sum)
  {
    float mw = m_own;
    if constexpr (LPK == 16) {
      if constexpr (HL <= 1) mw = fmaxf(mw, dpp_mov<kDppRowRor + 1>(mw));
      if constexpr (HL <= 2) mw = fmaxf(mw, dpp_mov<kDppRowRor + 2>(mw));
      if constexpr (HL <= 4) mw = fmaxf(mw, dpp_mov<kDppRowRor + 4>(mw));
      mw = fmaxf(mw, dpp_mov<kDppRowRor + 8>(mw));
    } else {
      if constexpr (HL <= 1) mw = fmaxf(mw, quad_xor<1>(mw));
      if constexpr (HL <= 2) mw = fmaxf(mw, quad_xor<2>(mw));
      if constexpr (HL <= 4) mw = fmaxf(mw, __shfl_xor(mw, 4));
      mw = fmaxf(mw, dpp_mov<kDppRowRor + 8>(mw));
    }
    mw = fmaxf(mw, __shfl_xor(mw, 16));
    mw = fmaxf(mw, __shfl_xor(mw, 32));
    // every owner set of a head saw the same keys, so their m_own and l_own are identical copies:
    // only the key groups differ.  Scale to the wave's reference and add up the key groups.
    const float cf = (m_own == -INFINITY) ? 0.f : fast_exp2(m_own - mw);
    float cf_o = 0.f;
    if constexpr (HL == 8) cf_o = dpp_mov<kDppHalfMirror>(cf);
    float cfs[HL];
    cfs[0] = cf;
    if constexpr (HL >= 2) cfs[1] = quad_xor<1>(cf);
    if constexpr (HL >= 4) { cfs[2] = quad_xor<2>(cf); cfs[3] = quad_xor<3>(cf); }
    if constexpr (HL == 8) {
      cfs[4] = cf_o; cfs[5] = quad_xor<1>(cf_o); cfs[6] = quad_xor<2>(cf_o); cfs[7] = quad_xor<3>(cf_o);
    }
    l_own = across_groups_sum<LPK>(l_own * cf);
    m_own = mw;
#pragma unroll
    for (int k = 0; k < HL; ++k)
#pragma unroll
      for (int vi = 0; vi < VPL; ++vi)
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[k][vi][e] = across_groups_sum<LPK>(acc[k][vi][e] * cfs[k]);
  }

  // wave partial -> LDS -> work-group partial
  __shared__ float sm_acc[kWaves][HL][D];
  __shared__ float sm_m[kWaves][HL];
  __shared__ float sm_l[kWaves][HL];
  if (kg == 0) {
#pragma unroll
    for (int k = 0; k < HL; ++k)
#pragma unroll
      for (int vi = 0; vi < VPL; ++vi)
#pragma unroll
        for (int e = 0; e < EPV; ++e) sm_acc[wave][hm ^ k][(vi * LPK + c) * EPV + e] = acc[k][vi][e];
    if (c < HL) {
      sm_m[wave][hm] = m_own;
      sm_l[wave][hm] = l_own;
    }
  }
  __syncthreads();

  for (int idx = tid; idx < HL * D; idx += kThreads) {
    const int h = idx / D, d = idx - h * D;
    const int hl = pass * HL + h;
    if (hl >= s.G) continue;
    float mx = sm_m[0][h];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, sm_m[w][h]);
    float o = 0.f, lt = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float wgt = fast_exp2(sm_m[w][h] - mx);  // a wave without tiles has reference -inf -> 0
      o = fmaf(wgt, sm_acc[w][h][d], o);
      lt = fmaf(wgt, sm_l[w][h], lt);
    }
    const size_t slot = ((size_t)b * s.H + (g * s.G + hl)) * s.S_max + split;
    a.sc.part_o[slot * D + d] = o;
    if (d == 0) {
      a.sc.part_ml[slot * 2] = mx;
      a.sc.part_ml[slot * 2 + 1] = lt;
    }
  }
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

struct FinishArgs {
  Shape s;
  LayerView lv;
  Scratch sc;
  void* out;
  SeqMask mask;
  float inv_H;
};

constexpr int kFinishThreads = 256;

// grid (H + ceil(max n_d / 256), B).  Blocks x < H merge the split partials of head x and write
// Att_t (Eq. 2).  The other blocks own 256 decode slots each: they rebuild every head's softmax
// normaliser from the split (max, sum) pairs, turn the stashed logits into probabilities, take the
// head mean (Eq. 4) and apply I <- alpha*I + abar (Eq. 5), with I = 0 for the new slot (Eq. 6).
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

// Softmax normaliser of one head from its split (reference, sum) pairs, by one whole wave:
// returns the common reference mx and the total sum L relative to it (both base 2).
__device__ __forceinline__ void wave_merge_ml(const float* ml, int ns, int lane, float& mx, float& L) {
  float m_loc = -INFINITY;
  for (int i = lane; i < ns; i += 64) m_loc = fmaxf(m_loc, ml[2 * i]);
  mx = wave_max(m_loc);
  float l_loc = 0.f;
  for (int i = lane; i < ns; i += 64) l_loc = fmaf(fast_exp2(ml[2 * i] - mx), ml[2 * i + 1], l_loc);
  L = wave_sum(l_loc);
}

template <int D>
__global__ __launch_bounds__(kFinishThreads) void finish_kernel(const FinishArgs a) {
  const Shape& s = a.s;
  const int b = blockIdx.y;
  if (!a.mask.active(b)) return;
  const int M = a.lv.mlen[b];
  const int n1 = a.lv.nd_eff[b];
  const int n0 = n1 - 1;
  const int ns = (M + s.CH - 1) / s.CH + (n1 + s.CH - 1) / s.CH;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  extern __shared__ float smem[];  // head blocks: [S_max] split weights; slot blocks: [H] normalisers

  if ((int)blockIdx.x < s.H) {
    const int h = blockIdx.x;
    constexpr int SUB = kFinishThreads / D;  // split subsets summed in parallel
    const int d = tid % D, sub = tid / D;
    const size_t slot0 = ((size_t)b * s.H + h) * s.S_max;
    const float* ml = a.sc.part_ml + slot0 * 2;
    float mx, L;
    wave_merge_ml(ml, ns, lane, mx, L);        // every wave computes the same pair
    for (int i = tid; i < ns; i += kFinishThreads) smem[i] = fast_exp2(ml[2 * i] - mx);
    __syncthreads();
    float o0 = 0.f, o1 = 0.f;
    const float* po = a.sc.part_o + slot0 * D + d;
    int i = sub;
    for (; i + SUB < ns; i += 2 * SUB) {       // two independent loads in flight
      o0 = fmaf(smem[i], po[(size_t)i * D], o0);
      o1 = fmaf(smem[i + SUB], po[(size_t)(i + SUB) * D], o1);
    }
    if (i < ns) o0 = fmaf(smem[i], po[(size_t)i * D], o0);
    __shared__ float red[kFinishThreads];
    red[tid] = o0 + o1;
    __syncthreads();
    if (sub == 0) {
      float o = red[d];
#pragma unroll
      for (int k = 1; k < SUB; ++k) o += red[k * D + d];
      const float r = o / L;
      const size_t oi = ((size_t)b * s.H + h) * D + d;
      if (s.bf16) ((uint16_t*)a.out)[oi] = f32_to_bf16_rne(r);
      else ((float*)a.out)[oi] = r;
    }
    if (tid == 0) {
      a.sc.lse[b * s.H + h] = mx + log2f(L);
      if (h == 0) a.lv.nd[b] = n1;  // the append becomes visible to the next kernel
    }
    return;
  }

  const int jb = ((int)blockIdx.x - s.H) * kFinishThreads;
  if (jb >= n1) return;
  for (int h = wave; h < s.H; h += kFinishThreads / 64) {
    float mx, L;
    wave_merge_ml(a.sc.part_ml + ((size_t)b * s.H + h) * s.S_max * 2, ns, lane, mx, L);
    if (lane == 0) smem[h] = mx + log2f(L);
  }
  __syncthreads();
  const int j = jb + tid;
  if (j >= n1) return;
  float sum0 = 0.f, sum1 = 0.f;
  const float* lg = a.sc.logits + (size_t)b * s.H * s.cap + j;
  int h = 0;
  for (; h + 1 < s.H; h += 2) {
    sum0 += fast_exp2(lg[(size_t)h * s.cap] - smem[h]);
    sum1 += fast_exp2(lg[(size_t)(h + 1) * s.cap] - smem[h + 1]);
  }
  if (h < s.H) sum0 += fast_exp2(lg[(size_t)h * s.cap] - smem[h]);
  const float abar = (sum0 + sum1) * a.inv_H;
  const size_t si = (size_t)b * s.cap + j;
  const float prev = (j == n0) ? 0.f : a.lv.score[si];
  a.lv.score[si] = fmaf(s.alpha, prev, abar);
  a.sc.abar[si] = abar;
  if (j == n0) {
    const int t = a.lv.tpos[b];
    a.lv.pos[si] = t;
    a.lv.tpos[b] = t + 1;
  }
}

template <bool BF16, int D, int HL, int IT, int WPB, bool PF, bool DIAG = false>
hipError_t launch_attn_v(const AttnArgs& a, dim3 grid, hipStream_t st) {
  constexpr int NV = D * (BF16 ? 2 : 4) / 16;
  constexpr int LPK = NV < 16 ? NV : 16;
  hipLaunchKernelGGL((attn_split_kernel<BF16, D, HL, LPK, IT, WPB, PF, DIAG>), grid, dim3(WPB * 64), 0, st, a);
  return hipGetLastError();
}

// Tile depth, work-group size and prefetch.  Variant 0 is the tuned default; the others exist for
// tuning runs on the Llama/Qwen-shaped bf16 kernels only.
template <bool BF16, int D, int HL>
hipError_t launch_attn_t(const AttnArgs& a, dim3 grid, hipStream_t st) {
  if constexpr (BF16 && D == 128 && (HL == 4 || HL == 8)) {
    switch (a.s.variant) {
      case 1: return launch_attn_v<BF16, D, HL, 4, 4, true>(a, grid, st);
      case 2: return launch_attn_v<BF16, D, HL, 2, 4, true>(a, grid, st);
      case 3: return launch_attn_v<BF16, D, HL, 4, 4, false>(a, grid, st);
      case 4: return launch_attn_v<BF16, D, HL, 2, 4, false>(a, grid, st);
      case 5: return launch_attn_v<BF16, D, HL, 8, 4, false>(a, grid, st);
      case 6: return launch_attn_v<BF16, D, HL, 8, 4, true>(a, grid, st);
      case 7: return launch_attn_v<BF16, D, HL, 4, 8, true>(a, grid, st);
      case 8: return launch_attn_v<BF16, D, HL, 2, 8, true>(a, grid, st);
      case 9: return launch_attn_v<BF16, D, HL, 4, 2, true>(a, grid, st);
      case 10: return launch_attn_v<BF16, D, HL, 4, 4, true, true>(a, grid, st);
      case 11: return launch_attn_v<BF16, D, HL, 4, 4, false, true>(a, grid, st);
      case 12: return launch_attn_v<BF16, D, HL, 8, 4, false, true>(a, grid, st);
      default: break;
    }
  }
  return launch_attn_v<BF16, D, HL, 4, 4, true>(a, grid, st);
}

template <bool BF16, int D>
hipError_t launch_attn_d(const AttnArgs& a0, hipStream_t st, int grid_splits) {
  AttnArgs a = a0;
  const int G = a.s.G;
  const int hl = (G == 1) ? 1 : (G == 2) ? 2 : (G <= 4) ? 4 : 8;  // head lanes per key group
  a.passes = (G + hl - 1) / hl;
  dim3 grid(grid_splits, a.s.Hkv * a.passes, a.s.B);
  switch (hl) {
    case 1: return launch_attn_t<BF16, D, 1>(a, grid, st);
    case 2: return launch_attn_t<BF16, D, 2>(a, grid, st);
    case 4: return launch_attn_t<BF16, D, 4>(a, grid, st);
    default: return launch_attn_t<BF16, D, 8>(a, grid, st);
  }
}

}  // namespace

hipError_t launch_attn(const Shape& s, const LayerView& lv, const Scratch& sc, const void* q,
                       const void* k_new, const void* v_new, const SeqMask& mask, int grid_splits,
                       hipStream_t st) {
  AttnArgs a;
  a.s = s; a.lv = lv; a.sc = sc;
  a.q = (const char*)q; a.k_new = (const char*)k_new; a.v_new = (const char*)v_new;
  a.mask = mask; a.passes = 1;
  if (s.bf16) return s.D == 128 ? launch_attn_d<true, 128>(a, st, grid_splits) : launch_attn_d<true, 64>(a, st, grid_splits);
  return s.D == 128 ? launch_attn_d<false, 128>(a, st, grid_splits) : launch_attn_d<false, 64>(a, st, grid_splits);
}

hipError_t launch_finish(const Shape& s, const LayerView& lv, const Scratch& sc, void* out,
                         const SeqMask& mask, int max_nd_eff, hipStream_t st) {
  FinishArgs a;
  a.s = s; a.lv = lv; a.sc = sc; a.out = out; a.mask = mask; a.inv_H = 1.0f / (float)s.H;
  dim3 grid(s.H + (max_nd_eff + kFinishThreads - 1) / kFinishThreads, s.B);
  const size_t smem = (size_t)(s.H > s.S_max ? s.H : s.S_max) * sizeof(float);
  if (s.D == 128) hipLaunchKernelGGL((finish_kernel<128>), grid, dim3(kFinishThreads), smem, st, a);
  else hipLaunchKernelGGL((finish_kernel<64>), grid, dim3(kFinishThreads), smem, st, a);
  return hipGetLastError();
}

}  // namespace mkv
