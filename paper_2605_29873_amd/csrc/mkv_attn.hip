// Split-K single-query attention over (prefill pool U decode pool) with logit emission for the
// decode keys, and the finishing kernel that merges the splits, writes Att_t and applies the
// head-mean + momentum update.  Paper: KV-cache preliminaries Eq. 2; Moment-KV Eq. 4-6;
// Algorithm 1 lines "append", "Softmax", "Mean", slice, and the importance loop.
//
// gfx950 only.  One wavefront = 64 lanes.  No matrix cores: per KV byte there are only G
// multiply-adds (G = query heads per KV head), so the kernel is a bandwidth-bound stream over K
// and V with the arithmetic on the vector ALU.
#include "mkv_internal.h"
#include "mkv_device.h"

#include <hip/hip_ext.h>

#include <math.h>
#include <string.h>

#include <type_traits>

namespace mkv {
namespace {

using namespace dev;


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
  int R;       // keys per work-group: the flattened key axis is cut into equal ranges
  int* occupancy;  // host pointer, only for the occupancy query
};

// Work-group k streams the keys [k*R, (k+1)*R) of the FLATTENED key axis -- sequence by sequence,
// inside a sequence unit by unit (unit = one KV head x one pass of up to HL of its query heads),
// inside a unit the prefill pool and then the decode pool -- so every work-group moves the same
// number of bytes whatever the mix of sequence lengths, and the launch is exactly as many
// work-groups as the chip holds at once.  For every unit its range touches ("piece") it leaves an
// un-normalised partial (reference, sum, sum p*V) per head in slot  k + unit index,  which keeps
// the slots of one unit contiguous.
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
template <bool BF16, int D, int HL, int LPK, int IT, int WPB, int NBUF>
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
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int c = lane % LPK;
  const int kg = lane / LPK;
  const int units = s.Hkv * s.passes;

  __shared__ long long offs[kMaxBatch + 1];
  __shared__ float sm_acc[kWaves][HL][D];
  __shared__ float sm_m[kWaves][HL];
  __shared__ float sm_l[kWaves][HL];
  constexpr int WT = 6144 / (HL * TK);   // decode tiles per logit staging window (24 KiB of LDS)
  constexpr int SK = WT * TK;            // keys per window
  __shared__ float sm_logit[HL][SK];
  if (wave == 0) build_offsets(s, a.lv, a.mask, units, 1 + unit_extra(s), offs, lane);
  else if (wave == 1) warm_kernel_arguments<sizeof(AttnArgs)>();   // meanwhile, for all waves of the compute unit
  __syncthreads();
  if (blockIdx.x == 0) {  // bookkeeping for the finishing kernel
    for (int b = tid; b <= s.B; b += kThreads) {
      a.sc.offs[b] = offs[b];
      if (b < s.B && a.mask.active(b)) {
        a.lv.nd_eff[b] = a.lv.nd[b] + 1;
        for (int sv = 0; sv < s.S; ++sv) a.sc.evict_key[b * s.S + sv] = ~0ull;   // this step's selection may land here
      }
    }
  }
  const long long total = offs[s.B];
  long long r0 = (long long)blockIdx.x * a.R;
  const long long r1 = min(total, r0 + a.R);
  if (r0 >= r1) return;

  // sequence that holds key r0: last b with offs[b] <= r0 (inactive sequences have empty spans)
  int b;
  {
    int lo = 0, hi = s.B;  // invariant: offs[lo] <= r0 < offs[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (offs[mid] <= r0) lo = mid; else hi = mid;
    }
    b = lo;
  }

  // head owned by this lane, as coordinates in the exchange basis (see above)
  int hm;
  if constexpr (HL == 8) {
    const int i = c & 7, hi = i >> 2;
    hm = (hi << 2) | ((((i >> 1) & 1) ^ hi) << 1) | ((i & 1) ^ hi);
  } else {
    hm = c & (HL - 1);
  }

  while (r0 < r1) {
    while (offs[b + 1] <= r0) ++b;      // skip to the sequence of r0 (spans of inactive ones are empty)
    const int M = a.lv.mlen[b];
    const int n0 = a.lv.nd[b];
    const int n1 = n0 + 1;              // the pool the softmax sees includes the token appended now
    const int L = M + n1;
    // On the flattened axis a unit is piece_pad positions longer than its L keys: the first ones
    // stand for what starting a piece costs, so that a work-group whose range crosses a unit
    // boundary gets that many keys fewer.  A range that ends inside them has no keys of the unit
    // and leaves no partial.
    const int Lp = L + unit_extra(s);                   // (and tail_pad positions behind the keys)
    const int ul = (int)((r0 - offs[b]) / Lp);          // unit inside the sequence
    const int g = ul / s.passes;
    const int pass = ul - g * s.passes;
    const int kav = (int)(r0 - offs[b] - (long long)ul * Lp);
    const int kev = (int)min((long long)Lp, kav + (r1 - r0));
    const int ka = min(max(kav - s.piece_pad, 0), L);   // first key of the piece in the unit
    const int ke = min(max(kev - s.piece_pad, 0), L);   // one past its last key
    if (ke <= ka) {
      r0 += kev - kav;
      continue;
    }
    // the piece as two sub-ranges: prefill keys [p0, p1), decode slots [d0, d1)
    const int p0 = min(ka, M), p1 = min(ke, M);
    const int d0 = max(ka, M) - M, d1 = max(ke, M) - M;
    const int ntp = (p1 - p0 + TK - 1) / TK;
    const int ntd = (d1 - d0 + TK - 1) / TK;
    const int ntile = ntp + ntd;
    // the new row: from k_new / v_new, or already in the pool when a producer kernel wrote it
    // there (k_new == nullptr): then no slot is special
    const int jnew = a.k_new ? n0 : -1;

    const size_t head_row = (size_t)b * s.Hkv + g;
    const char* kpre = (const char*)a.lv.Kp + head_row * (size_t)s.pstride * ROWB;
    const char* vpre = (const char*)a.lv.Vp + head_row * (size_t)s.pstride * ROWB;
    const char* kdec = (const char*)a.lv.Kd + head_row * (size_t)s.dstride * ROWB;
    const char* vdec = (const char*)a.lv.Vd + head_row * (size_t)s.dstride * ROWB;
    const char* knew = a.k_new + head_row * ROWB;
    const char* vnew = a.v_new + head_row * ROWB;

    // Append (Alg. 1: pool_d <- pool_d U {(K_t, V_t)}): the work-group whose piece holds the new
    // slot stores the row for later steps; in this step every reader takes it from k_new / v_new.
    if (pass == 0 && jnew >= d0 && jnew < d1 && tid < 2 * NV) {
      const int vsel = tid / NV, vec = tid - vsel * NV;
      const char* src = (vsel ? vnew : knew) + vec * 16;
      char* dst = (char*)(vsel ? a.lv.Vd : a.lv.Kd) + (head_row * (size_t)s.dstride + (size_t)jnew) * ROWB + vec * 16;
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
    float* const logit_base = a.sc.logits + ((size_t)b * s.H + g * s.G + pass * HL) * s.cap;
    const int heads_here = min(HL, s.G - pass * HL);     // real heads of this pass

    float m_own = -INFINITY, l_own = 0.f;
    float acc[HL][VPL][EPV];                             // acc[k] belongs to head hm ^ k
#pragma unroll
    for (int k = 0; k < HL; ++k)
#pragma unroll
      for (int vi = 0; vi < VPL; ++vi)
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[k][vi][e] = 0.f;

    auto load_tile = [&](int tt, uint4 (&kr)[IT][VPL], uint4 (&vr)[IT][VPL]) __attribute__((always_inline)) {
      const bool dec = tt >= ntp;
      const int jb = dec ? d0 + (tt - ntp) * TK : p0 + tt * TK;
      const int jl = (dec ? d1 : p1) - 1;
      const char* kbase = dec ? kdec : kpre;
      const char* vbase = dec ? vdec : vpre;
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int j = min(jb + it * KPW + kg, jl);  // clamp: masked later
        const bool isnew = dec && (j == jnew);
        const char* kp = isnew ? knew : kbase + (size_t)j * ROWB;
        const char* vp = isnew ? vnew : vbase + (size_t)j * ROWB;
#pragma unroll
        for (int vi = 0; vi < VPL; ++vi) {
          kr[it][vi] = ldg16_stream(kp + (vi * LPK + c) * 16);
          vr[it][vi] = ldg16_stream(vp + (vi * LPK + c) * 16);
        }
      }
    };

    // Logits of decode keys are staged in LDS, a window of SK keys at a time, and written out by
    // the whole work-group when the window (or the piece) ends.  Stores are kept out of the
    // streaming loop because loads and stores share one completion counter on this hardware: with
    // a store in the loop, every wait for a tile's loads would also wait for the prefetched tiles,
    // and waiting for a store's completion under full read load costs microseconds.
    int win = 0;   // current decode window of the piece

    // One tile: logits of IT keys per lane group, softmax update by the owner lanes, value
    // accumulation.  Each owner lane keeps its own running reference m_own, raised only when a
    // tile's maximum exceeds it by more than kSlack (base-2 units): exp2(s - m) then stays below
    // 2^kSlack, far from overflow, and the rescale is rare.  Lane groups are merged after the loop.
    constexpr float kSlack = 8.0f;
    auto compute_tile = [&](int tt, const uint4 (&kr)[IT][VPL], const uint4 (&vr)[IT][VPL]) __attribute__((always_inline)) {
      const bool dec = tt >= ntp;
      const int jb = dec ? d0 + (tt - ntp) * TK : p0 + tt * TK;
      const int jn = dec ? d1 : p1;
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
        // first owner lane of each head stages the logit; slot = key offset inside the window
        if (dec && c < HL) sm_logit[hm][(tt - ntp - win * WT) * TK + it * KPW + kg] = d;
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

    // NBUF register buffers per wave: the loads of the next NBUF-1 tiles are in flight while a
    // tile is being worked on (NBUF = 1: load, then compute).  The steady-state loop is unrolled
    // by NBUF so that every buffer index is a compile-time constant, and inside it the prefetch is
    // unconditional: a prefetch under an `if` would make the compiler wait for ALL outstanding
    // loads before every tile (it must assume the branch was not taken), which defeats it.
    auto run_tiles = [&](int t_lo, int t_hi) __attribute__((always_inline)) {
      uint4 kbuf[NBUF][IT][VPL], vbuf[NBUF][IT][VPL];
      int tt = t_lo + wave;
      if constexpr (NBUF == 1) {
        // the first tile's loads go out before the wait that clears earlier stores (and the query
        // loads), so that their latency overlaps with it
        const bool any = tt < t_hi;
        if (any) load_tile(tt, kbuf[0], vbuf[0]);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): no earlier store is pending inside the loop
        if (any) {
          compute_tile(tt, kbuf[0], vbuf[0]);
          tt += kWaves;
        }
        for (; tt < t_hi; tt += kWaves) {
          load_tile(tt, kbuf[0], vbuf[0]);
          compute_tile(tt, kbuf[0], vbuf[0]);
        }
      } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): no earlier store is pending inside the loop
        constexpr int AHEAD = (NBUF - 1) * kWaves;
#pragma unroll
        for (int u = 0; u < NBUF - 1; ++u)
          if (tt + u * kWaves < t_hi) load_tile(tt + u * kWaves, kbuf[u], vbuf[u]);
        // tiles still buffered when the steady state ends, starting at buffer U
        auto drain = [&](auto U) __attribute__((always_inline)) {
#pragma unroll
          for (int i = 0; i < NBUF - 1; ++i) {
            if (tt < t_hi) {
              compute_tile(tt, kbuf[(decltype(U)::value + i) % NBUF], vbuf[(decltype(U)::value + i) % NBUF]);
              tt += kWaves;
            }
          }
        };
        int left_at = -1;
        while (left_at < 0) {
#pragma unroll
          for (int u = 0; u < NBUF; ++u) {
            if (tt + AHEAD >= t_hi) { left_at = u; break; }
            load_tile(tt + AHEAD, kbuf[(u + NBUF - 1) % NBUF], vbuf[(u + NBUF - 1) % NBUF]);
            compute_tile(tt, kbuf[u], vbuf[u]);
            tt += kWaves;
          }
        }
        if (left_at == 0) drain(std::integral_constant<int, 0>{});
        if constexpr (NBUF >= 2) { if (left_at == 1) drain(std::integral_constant<int, 1>{}); }
        if constexpr (NBUF >= 3) { if (left_at == 2) drain(std::integral_constant<int, 2>{}); }
        if constexpr (NBUF >= 4) { if (left_at == 3) drain(std::integral_constant<int, 3>{}); }
        static_assert(NBUF <= 4, "drain cases");
      }
    };

    // phases: all prefill tiles plus the first decode window, then one decode window per phase
    for (int t_lo = 0; t_lo < ntile; ++win) {
      const int t_hi = min(ntile, ntp + (win + 1) * WT);
      run_tiles(t_lo, t_hi);
      const int wk0 = win * SK;                       // window start, in keys after d0
      const int nk = min(d1 - d0 - wk0, SK);          // staged keys (<= 0: no decode key yet)
      if (nk > 0) {
        __syncthreads();
        for (int h = 0; h < heads_here; ++h)
          for (int key = tid; key < nk; key += kThreads)
            logit_base[(size_t)h * s.cap + d0 + wk0 + key] = sm_logit[h][key];
        if (t_hi < ntile) {
          __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0) before the window is reused
          __syncthreads();
        }
      }
      t_lo = t_hi;
    }

    // merge the lane sets of the wave: common reference per head, then sums across key groups
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
      // the owner sets of a head inside one key group saw the same keys and hold identical copies
      // of m_own and l_own: only the key groups differ.  Scale to the wave's reference and add up
      // the key groups.
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

    // wave partial -> LDS -> work-group partial of this piece
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
    const size_t slot = (size_t)blockIdx.x + (size_t)b * units + ul;
    for (int idx = tid; idx < HL * D; idx += kThreads) {
      const int h = idx / D, d = idx - h * D;
      float mx = sm_m[0][h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, sm_m[w][h]);
      float o = 0.f, lt = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        // a wave without tiles has reference -inf; if no wave had a tile, mx is -inf as well
        const float wgt = (sm_m[w][h] == -INFINITY) ? 0.f : fast_exp2(sm_m[w][h] - mx);
        o = fmaf(wgt, sm_acc[w][h][d], o);
        lt = fmaf(wgt, sm_l[w][h], lt);
      }
      a.sc.part_o[(slot * HL + h) * D + d] = o;
      if (d == 0) {
        a.sc.part_ml[(slot * HL + h) * 2] = mx;
        a.sc.part_ml[(slot * HL + h) * 2 + 1] = lt;
      }
    }
    __syncthreads();  // the LDS staging is reused by the next piece
    r0 += kev - kav;
  }
}

struct FinishArgs {
  Shape s;
  LayerView lv;
  Scratch sc;
  void* out;
  SeqMask mask;
  float inv_H;
  int R;  // keys per attention work-group of the launch being finished
};

constexpr int kFinishThreads = 256;

// Where the attention kernel left the partials of query head h of sequence b: first slot, number
// of slots, and the head's position inside a slot.
struct PieceSpan { size_t slot0; int ns; int hs; };
__device__ __forceinline__ PieceSpan piece_span(const Shape& s, const long long* offs, int R, int b, int h, int L) {
  const int g = h / s.G, hl = h - g * s.G;
  const int pass = hl / s.HL;
  const int ul = g * s.passes + pass;
  // a unit takes L + piece_pad + tail_pad positions of the flattened axis, its keys after piece_pad
  const long long off_u = offs[b] + (long long)ul * (L + unit_extra(s)) + s.piece_pad;
  const long long kf = off_u / R, kl = (off_u + L - 1) / R;
  PieceSpan p;
  p.slot0 = (size_t)kf + (size_t)b * s.Hkv * s.passes + ul;
  p.ns = (int)(kl - kf) + 1;
  p.hs = hl - pass * s.HL;
  return p;
}

// grid (H + ceil(max n_d / 256), B).  Blocks x < H merge the partials of head x and write Att_t
// (Eq. 2).  The other blocks own 256 decode slots each: they rebuild every head's softmax
// normaliser from the (reference, sum) pairs, turn the stashed logits into probabilities, take the
// head mean (Eq. 4) and apply I <- alpha*I + abar (Eq. 5), with I = 0 for the new slot (Eq. 6).
template <int D>
__global__ __launch_bounds__(kFinishThreads) void finish_kernel(const FinishArgs a) {
  warm_kernel_arguments<sizeof(FinishArgs)>();
  const Shape& s = a.s;
  const int b = blockIdx.y;
  if (!a.mask.active(b)) return;
  const int M = a.lv.mlen[b];
  const int n1 = a.lv.nd_eff[b];
  const int n0 = n1 - 1;
  const int Lb = M + n1;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mlstride = s.HL * 2;
  extern __shared__ float smem[];  // head blocks: piece weights; slot blocks: [H] normalisers

  if ((int)blockIdx.x < s.H) {
    const int h = blockIdx.x;
    constexpr int SUB = kFinishThreads / D;  // piece subsets summed in parallel
    const int d = tid % D, sub = tid / D;
    const PieceSpan sp = piece_span(s, a.sc.offs, a.R, b, h, Lb);
    const int ns = sp.ns;
    const float* ml = a.sc.part_ml + (sp.slot0 * s.HL + sp.hs) * 2;
    float mx, L;
    wave_merge_ml(ml, mlstride, ns, lane, mx, L);   // every wave computes the same pair
    for (int i = tid; i < ns; i += kFinishThreads) smem[i] = fast_exp2(ml[(size_t)i * mlstride] - mx);
    __syncthreads();
    float o0 = 0.f, o1 = 0.f;
    const float* po = a.sc.part_o + (sp.slot0 * s.HL + sp.hs) * D + d;
    const size_t ostride = (size_t)s.HL * D;
    int i = sub;
    for (; i + SUB < ns; i += 2 * SUB) {       // two independent loads in flight
      o0 = fmaf(smem[i], po[(size_t)i * ostride], o0);
      o1 = fmaf(smem[i + SUB], po[(size_t)(i + SUB) * ostride], o1);
    }
    if (i < ns) o0 = fmaf(smem[i], po[(size_t)i * ostride], o0);
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
  // Normalisers of all H heads, with the threads spread over (head, piece subset) so that the
  // (reference, sum) pairs of every head are fetched in one round of loads: `parts` threads per
  // head, partial maxima and sums combined through LDS.  smem: [H] normalisers, then 2 x [parts][hc].
  {
    const int hc = min(s.H, kFinishThreads);              // heads per round
    const int parts = kFinishThreads / hc;
    float* red = smem + s.H;
    for (int h0 = 0; h0 < s.H; h0 += hc) {
      const int hh = tid % hc, part = tid / hc;
      const int h = h0 + hh;
      const bool on = part < parts && h < s.H;
      PieceSpan sp = {0, 0, 0};
      const float* ml = a.sc.part_ml;
      float m_loc = -INFINITY;
      if (on) {
        sp = piece_span(s, a.sc.offs, a.R, b, h, Lb);
        ml = a.sc.part_ml + (sp.slot0 * s.HL + sp.hs) * 2;
        for (int i = part; i < sp.ns; i += parts) m_loc = fmaxf(m_loc, ml[(size_t)i * mlstride]);
        red[part * hc + hh] = m_loc;
      }
      __syncthreads();
      float mx = -INFINITY, l_loc = 0.f;
      if (on) {
        for (int p = 0; p < parts; ++p) mx = fmaxf(mx, red[p * hc + hh]);
        for (int i = part; i < sp.ns; i += parts)
          l_loc = fmaf(fast_exp2(ml[(size_t)i * mlstride] - mx), ml[(size_t)i * mlstride + 1], l_loc);
      }
      __syncthreads();
      if (on) red[part * hc + hh] = l_loc;
      __syncthreads();
      if (on && part == 0) {
        float L = 0.f;
        for (int p = 0; p < parts; ++p) L += red[p * hc + hh];
        smem[h] = mx + log2f(L);
      }
      __syncthreads();
    }
  }
  const int j = jb + tid;
  // When the step will evict exactly one token (the paper's cadence: trigger = budget and the pool
  // has just grown to budget + 1), the selection of Eq. 8 is an arg-min over the scores computed
  // right here: every slot block merges its candidates' minimum into the vector's evict_key.
  // One score vector per sequence (mean over all H heads, Eq. 4 as printed) or one per KV head
  // (mean over the G heads of the group): vector sv covers heads [sv*Hs, (sv+1)*Hs).
  const int Hs = s.H / s.S;
  const float inv_Hs = 1.0f / (float)Hs;
  const bool pick_one = s.trigger == s.budget && n1 == s.budget + 1;
  __shared__ unsigned long long key_slots[4];
  for (int sv = 0; sv < s.S; ++sv) {
    unsigned long long key = ~0ull;
    if (j < n1) {
      float sum0 = 0.f, sum1 = 0.f;
      const float* lg = a.sc.logits + ((size_t)b * s.H + (size_t)sv * Hs) * s.cap + j;
      const float* nq = smem + sv * Hs;
      int h = 0;
      for (; h + 15 < Hs; h += 16) {   // sixteen independent loads in flight
        float x[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) x[u] = lg[(size_t)(h + u) * s.cap];
#pragma unroll
        for (int u = 0; u < 16; u += 2) {
          sum0 += fast_exp2(x[u] - nq[h + u]);
          sum1 += fast_exp2(x[u + 1] - nq[h + u + 1]);
        }
      }
      for (; h + 3 < Hs; h += 4) {
        const float x0 = lg[(size_t)h * s.cap], x1 = lg[(size_t)(h + 1) * s.cap];
        const float x2 = lg[(size_t)(h + 2) * s.cap], x3 = lg[(size_t)(h + 3) * s.cap];
        sum0 += fast_exp2(x0 - nq[h]) + fast_exp2(x2 - nq[h + 2]);
        sum1 += fast_exp2(x1 - nq[h + 1]) + fast_exp2(x3 - nq[h + 3]);
      }
      for (; h < Hs; ++h) sum0 += fast_exp2(lg[(size_t)h * s.cap] - nq[h]);
      const float abar = (sum0 + sum1) * inv_Hs;
      const size_t si = ((size_t)b * s.S + sv) * s.cap + j;
      const float prev = (j == n0) ? 0.f : a.lv.score[si];
      const float I = fmaf(s.alpha, prev, abar);
      a.lv.score[si] = I;
      a.sc.abar[si] = abar;
      if (j == n0) a.lv.pos[si] = a.lv.tpos[b];
      if (pick_one && j < n1 - s.window) key = evict_key_of(I, j);
    }
    if (pick_one) block_min_key_to(key, a.sc.evict_key + b * s.S + sv, key_slots, tid);
  }
  if (j == n0) a.lv.tpos[b] += 1;
}

// grid.x == 0 asks how many work-groups of the variant fit on one compute unit (*a.occupancy).
// With `tm`, the launch carries start/stop events that time the kernel alone.
template <bool BF16, int D, int HL, int IT, int WPB, int NBUF>
hipError_t launch_attn_v(const AttnArgs& a, dim3 grid, hipStream_t st, const KernelTimer* tm) {
  constexpr int NV = D * (BF16 ? 2 : 4) / 16;
  constexpr int LPK = NV < 16 ? NV : 16;
  auto kern = attn_split_kernel<BF16, D, HL, LPK, IT, WPB, NBUF>;
  if (grid.x == 0) return hipOccupancyMaxActiveBlocksPerMultiprocessor(a.occupancy, kern, WPB * 64, 0);
  if (tm) hipExtLaunchKernelGGL(kern, grid, dim3(WPB * 64), 0, st, tm->start, tm->stop, 0, a);
  else hipLaunchKernelGGL(kern, grid, dim3(WPB * 64), 0, st, a);
  return hipGetLastError();
}

// Keys per lane group and tile, waves per work-group, register buffers.  Variant 0 is the tuned
// default; the others exist for tuning runs on the Llama/Qwen-shaped bf16 kernels (all of them
// compute the same result).
template <bool BF16, int D, int HL>
hipError_t launch_attn_t(const AttnArgs& a, dim3 grid, hipStream_t st, const KernelTimer* tm) {
  if constexpr (BF16 && D == 128 && (HL == 4 || HL == 8)) {
    switch (a.s.variant) {
      case 1: return launch_attn_v<BF16, D, HL, 4, 4, 1>(a, grid, st, tm);
      case 2: return launch_attn_v<BF16, D, HL, 4, 4, 2>(a, grid, st, tm);
      case 3: return launch_attn_v<BF16, D, HL, 2, 4, 2>(a, grid, st, tm);
      case 4: return launch_attn_v<BF16, D, HL, 2, 8, 1>(a, grid, st, tm);
      case 5: return launch_attn_v<BF16, D, HL, 4, 8, 2>(a, grid, st, tm);
      case 6: return launch_attn_v<BF16, D, HL, 8, 4, 1>(a, grid, st, tm);
      case 7: return launch_attn_v<BF16, D, HL, 2, 8, 3>(a, grid, st, tm);
      case 8: return launch_attn_v<BF16, D, HL, 2, 8, 4>(a, grid, st, tm);
      case 9: return launch_attn_v<BF16, D, HL, 2, 8, 2>(a, grid, st, tm);
      case 10: return launch_attn_v<BF16, D, HL, 1, 8, 4>(a, grid, st, tm);
      default: break;
    }
  }
  // default: 4 keys per lane group and tile, 8 waves per work-group, no software prefetch (the
  // resident waves hide the load latency at least as well, and it keeps the register count down)
  return launch_attn_v<BF16, D, HL, 4, 8, 1>(a, grid, st, tm);
}

template <bool BF16, int D>
hipError_t launch_attn_d(const AttnArgs& a, hipStream_t st, int n_groups, const KernelTimer* tm) {
  dim3 grid(n_groups);
  switch (a.s.HL) {
    case 1: return launch_attn_t<BF16, D, 1>(a, grid, st, tm);
    case 2: return launch_attn_t<BF16, D, 2>(a, grid, st, tm);
    case 4: return launch_attn_t<BF16, D, 4>(a, grid, st, tm);
    default: return launch_attn_t<BF16, D, 8>(a, grid, st, tm);
  }
}

}  // namespace

hipError_t launch_attn(const Shape& s, const LayerView& lv, const Scratch& sc, const void* q,
                       const void* k_new, const void* v_new, const SeqMask& mask, int keys_per_group,
                       int n_groups, hipStream_t st, const KernelTimer* tm) {
  AttnArgs a;
  a.s = s; a.lv = lv; a.sc = sc;
  a.q = (const char*)q; a.k_new = (const char*)k_new; a.v_new = (const char*)v_new;
  a.mask = mask; a.R = keys_per_group; a.occupancy = nullptr;
  if (s.bf16) return s.D == 128 ? launch_attn_d<true, 128>(a, st, n_groups, tm) : launch_attn_d<true, 64>(a, st, n_groups, tm);
  return s.D == 128 ? launch_attn_d<false, 128>(a, st, n_groups, tm) : launch_attn_d<false, 64>(a, st, n_groups, tm);
}

hipError_t attn_groups_per_cu(const Shape& s, int* out) {
  AttnArgs a;
  memset(&a, 0, sizeof a);
  a.s = s; a.occupancy = out;
  if (s.bf16) return s.D == 128 ? launch_attn_d<true, 128>(a, nullptr, 0, nullptr) : launch_attn_d<true, 64>(a, nullptr, 0, nullptr);
  return s.D == 128 ? launch_attn_d<false, 128>(a, nullptr, 0, nullptr) : launch_attn_d<false, 64>(a, nullptr, 0, nullptr);
}

hipError_t launch_finish(const Shape& s, const LayerView& lv, const Scratch& sc, void* out,
                         const SeqMask& mask, int max_nd_eff, int keys_per_group, hipStream_t st,
                         const KernelTimer* tm) {
  FinishArgs a;
  a.s = s; a.lv = lv; a.sc = sc; a.out = out; a.mask = mask; a.inv_H = 1.0f / (float)s.H;
  a.R = keys_per_group;
  dim3 grid(s.H + (max_nd_eff + kFinishThreads - 1) / kFinishThreads, s.B);
  // head blocks: one weight per piece; slot blocks: H normalisers + a 256-entry reduction area
  const size_t smem = (size_t)(s.H + kFinishThreads > s.max_groups ? s.H + kFinishThreads : s.max_groups) * sizeof(float);
  auto kern = s.D == 128 ? finish_kernel<128> : finish_kernel<64>;
  if (tm) hipExtLaunchKernelGGL(kern, grid, dim3(kFinishThreads), smem, st, tm->start, tm->stop, 0, a);
  else hipLaunchKernelGGL(kern, grid, dim3(kFinishThreads), smem, st, a);
  return hipGetLastError();
}

}  // namespace mkv
