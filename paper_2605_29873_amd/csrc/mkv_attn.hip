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

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;

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
  int passes;  // ceil(G / GT): head passes per KV head
};

// Work-group (split, kv head x pass, seq): streams keys [j0, jn) of one segment (prefill or
// decode) of one KV head, for up to GT of its query heads, and leaves an un-normalised partial
// (max, sum, sum p*V) per head.  Lane layout: LPK adjacent lanes share a key, lane c of a group
// holding the 16-byte vectors c, c+LPK, ... of the row, so one load instruction of a wave reads
// 64/LPK rows x (LPK*16) contiguous bytes.
template <bool BF16, int D, int GT, int LPK, int IT>
__global__ __launch_bounds__(kThreads) void attn_split_kernel(const AttnArgs a) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int ROWB = D * ES;
  constexpr int NV = ROWB / 16;
  constexpr int VPL = NV / LPK;
  constexpr int EPV = 16 / ES;
  constexpr int KPW = 64 / LPK;
  constexpr int TK = KPW * IT;
  static_assert(NV % LPK == 0 && VPL >= 1, "row must split evenly over the lane group");

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

  const size_t head_row = (size_t)b * s.Hkv + g;
  const size_t pool_rows = dec ? (size_t)s.cap : (size_t)s.max_prefill;
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

  // queries of this pass, in storage form, at this lane's vector positions
  uint4 qv[GT][VPL];
  int hq[GT];
#pragma unroll
  for (int h = 0; h < GT; ++h) {
    const int hl = pass * GT + h;
    hq[h] = (hl < s.G) ? g * s.G + hl : -1;
#pragma unroll
    for (int vi = 0; vi < VPL; ++vi) {
      qv[h][vi] = (hq[h] >= 0) ? ldg16(a.q + ((size_t)b * s.H + hq[h]) * ROWB + (vi * LPK + c) * 16)
                               : make_uint4(0, 0, 0, 0);
    }
  }

  float m[GT], l[GT], acc[GT][VPL][EPV];
#pragma unroll
  for (int h = 0; h < GT; ++h) {
    m[h] = -INFINITY;
    l[h] = 0.f;
#pragma unroll
    for (int vi = 0; vi < VPL; ++vi)
#pragma unroll
      for (int e = 0; e < EPV; ++e) acc[h][vi][e] = 0.f;
  }

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

  uint4 kr[IT][VPL], vr[IT][VPL];
  if (wave < ntile) load_tile(wave, kr, vr);

  for (int tt = wave; tt < ntile; tt += kWaves) {
    uint4 kn[IT][VPL], vn[IT][VPL];
    const bool more = tt + kWaves < ntile;
    if (more) load_tile(tt + kWaves, kn, vn);  // prefetch: in flight during this tile's math

    const int jb = j0 + tt * TK;
    float sc[IT][GT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int j = jb + it * KPW + kg;
#pragma unroll
      for (int h = 0; h < GT; ++h) {
        float d = 0.f;
#pragma unroll
        for (int vi = 0; vi < VPL; ++vi) d = dot_vec<BF16>(kr[it][vi], qv[h][vi], d);
        d = group_sum<LPK>(d) * s.scale_log2;
        sc[it][h] = (j < jn) ? d : -INFINITY;
      }
      if (dec && c == 0 && j < jn) {
#pragma unroll
        for (int h = 0; h < GT; ++h)
          if (hq[h] >= 0) a.sc.logits[((size_t)b * s.H + hq[h]) * s.cap + j] = sc[it][h];
      }
    }

    // online softmax, one rescale per tile (skipped when the running max did not move)
#pragma unroll
    for (int h = 0; h < GT; ++h) {
      float tm = sc[0][h];
#pragma unroll
      for (int it = 1; it < IT; ++it) tm = fmaxf(tm, sc[it][h]);
      tm = across_groups_max<LPK>(tm);
      if (tm > m[h]) {
        const float cf = fast_exp2(m[h] - tm);
        l[h] *= cf;
#pragma unroll
        for (int vi = 0; vi < VPL; ++vi)
#pragma unroll
          for (int e = 0; e < EPV; ++e) acc[h][vi][e] *= cf;
        m[h] = tm;
      }
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
#pragma unroll
      for (int h = 0; h < GT; ++h) {
        const float p = fast_exp2(sc[it][h] - m[h]);
        l[h] += p;
#pragma unroll
        for (int vi = 0; vi < VPL; ++vi) axpy_vec<BF16>(p, vr[it][vi], acc[h][vi]);
      }
    }

    if (more) {
#pragma unroll
      for (int it = 0; it < IT; ++it)
#pragma unroll
        for (int vi = 0; vi < VPL; ++vi) {
          kr[it][vi] = kn[it][vi];
          vr[it][vi] = vn[it][vi];
        }
    }
  }

  // wave partial -> LDS -> work-group partial
  __shared__ float sm_acc[kWaves][GT][D];
  __shared__ float sm_m[kWaves][GT];
  __shared__ float sm_l[kWaves][GT];
#pragma unroll
  for (int h = 0; h < GT; ++h) {
    l[h] = across_groups_sum<LPK>(l[h]);
#pragma unroll
    for (int vi = 0; vi < VPL; ++vi)
#pragma unroll
      for (int e = 0; e < EPV; ++e) {
        const float v = across_groups_sum<LPK>(acc[h][vi][e]);
        if (kg == 0) sm_acc[wave][h][(vi * LPK + c) * EPV + e] = v;
      }
    if (lane == 0) {
      sm_m[wave][h] = m[h];
      sm_l[wave][h] = l[h];
    }
  }
  __syncthreads();

  for (int idx = tid; idx < GT * D; idx += kThreads) {
    const int h = idx / D, d = idx - h * D;
    const int hl = pass * GT + h;
    if (hl >= s.G) continue;
    float mx = sm_m[0][h];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, sm_m[w][h]);
    float o = 0.f, lt = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float wgt = fast_exp2(sm_m[w][h] - mx);  // a wave without tiles has max -inf -> 0
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
template <int D>
__global__ __launch_bounds__(kFinishThreads) void finish_kernel(const FinishArgs a) {
  const Shape& s = a.s;
  const int b = blockIdx.y;
  if (!a.mask.active(b)) return;
  const int M = a.lv.mlen[b];
  const int n1 = a.lv.nd_eff[b];
  const int n0 = n1 - 1;
  const int ns = (M + s.CH - 1) / s.CH + (n1 + s.CH - 1) / s.CH;
  const int tid = threadIdx.x;

  if ((int)blockIdx.x < s.H) {
    const int h = blockIdx.x;
    constexpr int SUB = kFinishThreads / D;  // split subsets summed in parallel
    const int d = tid % D, sub = tid / D;
    const size_t slot0 = ((size_t)b * s.H + h) * s.S_max;
    const float* ml = a.sc.part_ml + slot0 * 2;
    float mx = -INFINITY;
    for (int i = 0; i < ns; ++i) mx = fmaxf(mx, ml[2 * i]);
    float L = 0.f, o = 0.f;
    for (int i = 0; i < ns; ++i) L = fmaf(fast_exp2(ml[2 * i] - mx), ml[2 * i + 1], L);
    for (int i = sub; i < ns; i += SUB)
      o = fmaf(fast_exp2(ml[2 * i] - mx), a.sc.part_o[(slot0 + i) * D + d], o);
    __shared__ float red[kFinishThreads];
    red[tid] = o;
    __syncthreads();
    if (sub == 0) {
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
  extern __shared__ float sm_lse[];  // [H]
  for (int h = tid; h < s.H; h += kFinishThreads) {
    const float* ml = a.sc.part_ml + ((size_t)b * s.H + h) * s.S_max * 2;
    float mx = -INFINITY;
    for (int i = 0; i < ns; ++i) mx = fmaxf(mx, ml[2 * i]);
    float L = 0.f;
    for (int i = 0; i < ns; ++i) L = fmaf(fast_exp2(ml[2 * i] - mx), ml[2 * i + 1], L);
    sm_lse[h] = mx + log2f(L);
  }
  __syncthreads();
  const int j = jb + tid;
  if (j >= n1) return;
  float sum = 0.f;
  const float* lg = a.sc.logits + (size_t)b * s.H * s.cap + j;
  for (int h = 0; h < s.H; ++h) sum += fast_exp2(lg[(size_t)h * s.cap] - sm_lse[h]);
  const float abar = sum * a.inv_H;
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

template <bool BF16, int D, int GT>
hipError_t launch_attn_t(const AttnArgs& a, dim3 grid, hipStream_t st) {
  // lanes per key / keys per lane per tile: chosen to keep the register count near 128
  constexpr int ROWB = D * (BF16 ? 2 : 4);
  constexpr int LPK = (ROWB / 16 >= 16) ? 16 : ROWB / 16;
  constexpr int IT = 4;
  hipLaunchKernelGGL((attn_split_kernel<BF16, D, GT, LPK, IT>), grid, dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

template <bool BF16, int D>
hipError_t launch_attn_d(const AttnArgs& a0, hipStream_t st, int grid_splits) {
  AttnArgs a = a0;
  const int G = a.s.G;
  const int gt = (G == 1) ? 1 : (G == 2) ? 2 : (G <= 4) ? 4 : (G <= 7) ? 7 : 8;
  a.passes = (G + gt - 1) / gt;
  dim3 grid(grid_splits, a.s.Hkv * a.passes, a.s.B);
  switch (gt) {
    case 1: return launch_attn_t<BF16, D, 1>(a, grid, st);
    case 2: return launch_attn_t<BF16, D, 2>(a, grid, st);
    case 4: return launch_attn_t<BF16, D, 4>(a, grid, st);
    case 7: return launch_attn_t<BF16, D, 7>(a, grid, st);
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
  const size_t smem = (size_t)s.H * sizeof(float);
  if (s.D == 128) hipLaunchKernelGGL((finish_kernel<128>), grid, dim3(kFinishThreads), smem, st, a);
  else hipLaunchKernelGGL((finish_kernel<64>), grid, dim3(kFinishThreads), smem, st, a);
  return hipGetLastError();
}

}  // namespace mkv
