// Multi-query decode step on the matrix cores: q_len = Q query rows per sequence and step
// (chunked or speculative decoding), causal among the Q appended tokens.  With the G query heads
// that share a KV head, a pass has up to 16 rows (heads x query positions) against every key, so
// QK^T and PV are dense 16-wide contractions and run on MFMA.  Paper: Eq. 2 (attention over the
// prefill and decode pools), Eq. 4-6 (head mean and momentum, applied once per query row in order),
// Algorithm 1 "append".  bf16 storage and head_dim 128 only.
//
// gfx950 only: v_mfma_f32_16x16x32_bf16.  Operand layouts (lane l, r = l % 16, j = l / 16):
//   A[m][k] : lane holds m = r, k = 8j .. 8j+7      B[k][n] : lane holds n = r, k = 8j .. 8j+7
//   C[m][n] : lane holds n = r, m = 4j .. 4j+3
#include "mkv_internal.h"
#include "mkv_device.h"

#include <hip/hip_ext.h>

#include <math.h>
#include <string.h>

namespace mkv {
namespace {

using namespace dev;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kD = 128;
constexpr int kRowB = kD * 2;      // bytes per K or V row
constexpr int kNV = kRowB / 16;    // 16-byte vectors per row
constexpr int kTK = 32;            // keys per wave tile
constexpr int kSK = 384;           // decode keys per logit staging window
constexpr int kSKP = kSK + 4;      // padded LDS row: spreads the 16 rows over the banks
constexpr int kWT = kSK / kTK;     // tiles per window

struct MqArgs {
  Shape s;
  LayerView lv;
  Scratch sc;
  const char* q;
  const char* k_new;
  const char* v_new;
  SeqMask mask;
  int R;        // keys per work-group
  int Q;        // query rows per sequence
  int HP;       // query heads served per pass: min(G, 16 / Q)
  int passes;   // passes per KV head: ceil(G / HP)
};

__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4& v) { return __builtin_bit_cast(bf16x8_t, v); }

// Same partition of the flattened key axis as the single-query kernel: work-group k takes keys
// [k*R, (k+1)*R), a unit is one KV head x one pass, and every piece of a unit leaves a partial
// (reference, sum, sum p*V) per row in slot  k + unit index.  A unit has L = M + n_d + Q keys.
//
// One wave tile is 32 keys.  Scores: S^T = K * Q^T as two 16-key MFMA tiles, the K rows as the A
// operand (lane (r, j) loads the 16-byte vectors 4*iv + j of key r; the queries are loaded the same
// way, so both operands see the same permutation of the head dimension).  The C layout leaves lane
// (r, j) with the scores of query row r against keys 4j .. 4j+3 of each tile -- which, rounded to
// bf16, is exactly the B operand of  O^T = V^T * P^T  with the 32 keys as the contraction index.
// The V^T operand wants, per lane, one head-dim element of 8 keys: lane (r, j) loads vector r of
// the 8 keys it contracts and transposes 16-bit halves in registers (one byte-permute per dword).
// The accumulators then hold O[row r][8 * (4j + i) + dc] for chunk dc, i = 0..3.
template <int WPB>
__global__ __launch_bounds__(WPB * 64) void attn_mq_kernel(const MqArgs a) {
  constexpr int kThreads = WPB * 64;
  const Shape& s = a.s;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r16 = lane & 15;
  const int j4 = lane >> 4;
  const int Q = a.Q;
  const int units = s.Hkv * a.passes;

  __shared__ long long offs[kMaxBatch + 1];
  __shared__ float sm_logit[16][kSKP];
  __shared__ float sm_part[WPB / 2][34][64];   // a wave's accumulators, reference and sum, lane-major
  if (wave == 0) build_offsets(s, a.lv, a.mask, units, Q, offs, lane);
  __syncthreads();
  if (blockIdx.x == 0) {
    for (int b = tid; b <= s.B; b += kThreads) {
      a.sc.offs[b] = offs[b];
      if (b < s.B && a.mask.active(b)) a.lv.nd_eff[b] = a.lv.nd[b] + Q;
    }
  }
  const long long total = offs[s.B];
  long long r0 = (long long)blockIdx.x * a.R;
  const long long r1 = min(total, r0 + a.R);
  if (r0 >= r1) return;

  int b;
  {
    int lo = 0, hi = s.B;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (offs[mid] <= r0) lo = mid; else hi = mid;
    }
    b = lo;
  }

  while (r0 < r1) {
    while (offs[b + 1] <= r0) ++b;
    const int M = a.lv.mlen[b];
    const int n0 = a.lv.nd[b];
    const int n1 = n0 + Q;
    const int L = M + n1;
    const int ul = (int)((r0 - offs[b]) / L);
    const int g = ul / a.passes;
    const int pass = ul - g * a.passes;
    const int ka = (int)(r0 - offs[b] - (long long)ul * L);
    const int ke = (int)min((long long)L, ka + (r1 - r0));
    const int p0 = min(ka, M), p1 = min(ke, M);
    const int d0 = max(ka, M) - M, d1 = max(ke, M) - M;
    const int ntp = (p1 - p0 + kTK - 1) / kTK;
    const int ntd = (d1 - d0 + kTK - 1) / kTK;
    const int ntile = ntp + ntd;
    const int nrows = min(a.HP, s.G - pass * a.HP) * Q;   // real rows of this pass

    const size_t head_row = (size_t)b * s.Hkv + g;
    const char* kpre = (const char*)a.lv.Kp + head_row * (size_t)s.pstride * kRowB;
    const char* vpre = (const char*)a.lv.Vp + head_row * (size_t)s.pstride * kRowB;
    const char* kdec = (const char*)a.lv.Kd + head_row * (size_t)s.dstride * kRowB;
    const char* vdec = (const char*)a.lv.Vd + head_row * (size_t)s.dstride * kRowB;
    // appended token qn of this KV head: row (b, qn, g) of k_new / v_new
    const size_t new_stride = (size_t)s.Hkv * kRowB;
    const char* knew = a.k_new + ((size_t)b * Q * s.Hkv + g) * kRowB;
    const char* vnew = a.v_new + ((size_t)b * Q * s.Hkv + g) * kRowB;

    // Append (Alg. 1): the work-group whose piece holds new slots stores their rows for later
    // steps; in this step every reader takes them from k_new / v_new.
    if (pass == 0) {
      const int a0 = max(d0, n0), a1 = min(d1, n1);
      for (int idx = tid; idx < (a1 - a0) * 2 * kNV; idx += kThreads) {
        const int row = idx / (2 * kNV), rem = idx - row * 2 * kNV;
        const int vsel = rem / kNV, vec = rem - vsel * kNV;
        const int jn = a0 + row;
        const char* src = (vsel ? vnew : knew) + (size_t)(jn - n0) * new_stride + vec * 16;
        char* dst = (char*)(vsel ? a.lv.Vd : a.lv.Kd) + (head_row * (size_t)s.dstride + (size_t)jn) * kRowB + vec * 16;
        *reinterpret_cast<uint4*>(dst) = ldg16(src);
      }
      if (g == 0) {
        const int t0 = a.lv.tpos[b];
        for (int idx = tid; idx < a1 - a0; idx += kThreads)
          a.lv.pos[(size_t)b * s.cap + a0 + idx] = t0 + (a0 + idx - n0);
      }
    }

    // query rows: row r = (head inside the pass) * Q + (query position)
    const int hl = r16 / Q, qi = r16 - hl * Q;
    uint4 qv[4];
    {
      const bool row_ok = r16 < nrows;
      const char* qp = a.q + (((size_t)b * Q + qi) * s.H + g * s.G + pass * a.HP + hl) * kRowB;
#pragma unroll
      for (int iv = 0; iv < 4; ++iv) qv[iv] = row_ok ? ldg16(qp + (4 * iv + j4) * 16) : make_uint4(0, 0, 0, 0);
    }
    float* const logit_base = a.sc.logits + ((size_t)b * s.H + g * s.G + pass * a.HP) * Q * s.cap;

    float m_run = -INFINITY, l_run = 0.f;   // m_run is identical in the four lanes of a row
    f32x4_t acc[8];
#pragma unroll
    for (int dc = 0; dc < 8; ++dc) acc[dc] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    auto load_tile = [&](int tt, uint4 (&kr)[2][4], uint4 (&vr)[2][4]) __attribute__((always_inline)) {
      const bool dec = tt >= ntp;
      const int jb = dec ? d0 + (tt - ntp) * kTK : p0 + tt * kTK;
      const int jl = (dec ? d1 : p1) - 1;
      const char* kbase = dec ? kdec : kpre;
      const char* vbase = dec ? vdec : vpre;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int jk = min(jb + 16 * h + r16, jl);          // clamp: masked later
        const bool knw = dec && jk >= n0;
        const char* kp = knw ? knew + (size_t)(jk - n0) * new_stride : kbase + (size_t)jk * kRowB;
#pragma unroll
        for (int iv = 0; iv < 4; ++iv) kr[h][iv] = ldg16(kp + (4 * iv + j4) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int jv = min(jb + 16 * h + 4 * j4 + i, jl);
          const bool vnw = dec && jv >= n0;
          const char* vp = vnw ? vnew + (size_t)(jv - n0) * new_stride : vbase + (size_t)jv * kRowB;
          vr[h][i] = ldg16(vp + r16 * 16);
        }
      }
    };

    int win = 0;
    constexpr float kSlack = 8.0f;
    auto compute_tile = [&](int tt, const uint4 (&kr)[2][4], const uint4 (&vr)[2][4]) __attribute__((always_inline)) {
      const bool dec = tt >= ntp;
      const int jb = dec ? d0 + (tt - ntp) * kTK : p0 + tt * kTK;
      const int jn = dec ? d1 : p1;
      float x[8];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        f32x4_t sv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int iv = 0; iv < 4; ++iv)
          sv = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kr[h][iv]), as_bf16x8(qv[iv]), sv, 0, 0, 0);
        const int key0 = jb + 16 * h + 4 * j4;
        float4 st;
        st.x = sv[0] * s.scale_log2; st.y = sv[1] * s.scale_log2;
        st.z = sv[2] * s.scale_log2; st.w = sv[3] * s.scale_log2;
        if (dec) *reinterpret_cast<float4*>(&sm_logit[r16][(tt - ntp - win * kWT) * kTK + 16 * h + 4 * j4]) = st;
        const float sx[4] = {st.x, st.y, st.z, st.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int key = key0 + i;
          // past the piece, or an appended token that comes after this row's own (causal order)
          const bool ok = key < jn && !(dec && key - n0 > qi);
          x[4 * h + i] = ok ? sx[i] : -INFINITY;
        }
      }
      float tm = x[0];
#pragma unroll
      for (int i = 1; i < 8; ++i) tm = fmaxf(tm, x[i]);
      if (__any(tm > m_run + kSlack)) {
        // the four lanes of a row raise the reference together, to the row's maximum over the tile
        tm = fmaxf(tm, __shfl_xor(tm, 16));
        tm = fmaxf(tm, __shfl_xor(tm, 32));
        if (tm > m_run + kSlack) {
          const float cf = fast_exp2(m_run - tm);   // exp2(-inf) = 0 on the first raise
          l_run *= cf;
          m_run = tm;
#pragma unroll
          for (int dc = 0; dc < 8; ++dc) acc[dc] *= cf;
        }
      }
      bf16x8_t pb;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float p = (x[i] == -INFINITY) ? 0.f : fast_exp2(x[i] - m_run);
        l_run += p;
        pb[i] = (__bf16)p;
      }
      // V^T operand for chunk dc: element 4h + i = bf16 number dc of the vector of key 4j + i, tile h
      uint32_t vw[2][4][4];
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          vw[h][i][0] = vr[h][i].x; vw[h][i][1] = vr[h][i].y; vw[h][i][2] = vr[h][i].z; vw[h][i][3] = vr[h][i].w;
        }
#pragma unroll
      for (int dc = 0; dc < 8; ++dc) {
        const int w = dc >> 1;
        const uint32_t sel = (dc & 1) ? 0x07060302u : 0x05040100u;   // high or low halves of both
        uint4 av;
        av.x = __builtin_amdgcn_perm(vw[0][1][w], vw[0][0][w], sel);
        av.y = __builtin_amdgcn_perm(vw[0][3][w], vw[0][2][w], sel);
        av.z = __builtin_amdgcn_perm(vw[1][1][w], vw[1][0][w], sel);
        av.w = __builtin_amdgcn_perm(vw[1][3][w], vw[1][2][w], sel);
        acc[dc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(av), pb, acc[dc], 0, 0, 0);
      }
    };

    auto run_tiles = [&](int t_lo, int t_hi) __attribute__((always_inline)) {
      uint4 kbuf[2][4], vbuf[2][4];
      int tt = t_lo + wave;
      const bool any = tt < t_hi;
      if (any) load_tile(tt, kbuf, vbuf);
      __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): no earlier store is pending inside the loop
      if (any) {
        compute_tile(tt, kbuf, vbuf);
        tt += WPB;
      }
      for (; tt < t_hi; tt += WPB) {
        load_tile(tt, kbuf, vbuf);
        compute_tile(tt, kbuf, vbuf);
      }
    };

    // phases: all prefill tiles plus the first decode window, then one decode window per phase;
    // the staged logits of a window are written out by the whole work-group
    for (int t_lo = 0; t_lo < ntile; ++win) {
      const int t_hi = min(ntile, ntp + (win + 1) * kWT);
      run_tiles(t_lo, t_hi);
      const int wk0 = win * kSK;
      const int nk = min(d1 - d0 - wk0, kSK);
      if (nk > 0) {
        __syncthreads();
        for (int r = 0; r < nrows; ++r)
          for (int key = tid; key < nk; key += kThreads)
            logit_base[(size_t)r * s.cap + d0 + wk0 + key] = sm_logit[r][key];
        if (t_hi < ntile) {
          __builtin_amdgcn_s_waitcnt(0x0F70);
          __syncthreads();
        }
      }
      t_lo = t_hi;
    }

    // the four lanes of a row saw different keys: add up their sums (the accumulators are already
    // contracted over all keys of the wave)
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);

    // waves -> one partial, halving the number of live waves per round
#pragma unroll
    for (int stride = WPB / 2; stride >= 1; stride >>= 1) {
      if (wave >= stride && wave < 2 * stride) {
        float (*dst)[64] = sm_part[wave - stride];
#pragma unroll
        for (int dc = 0; dc < 8; ++dc)
#pragma unroll
          for (int i = 0; i < 4; ++i) dst[dc * 4 + i][lane] = acc[dc][i];
        dst[32][lane] = m_run;
        dst[33][lane] = l_run;
      }
      __syncthreads();
      if (wave < stride) {
        float (*src)[64] = sm_part[wave];
        const float mo = src[32][lane], lo = src[33][lane];
        const float mx = fmaxf(m_run, mo);
        // a wave without visible keys has reference -inf
        const float wa = (m_run == -INFINITY) ? 0.f : fast_exp2(m_run - mx);
        const float wb = (mo == -INFINITY) ? 0.f : fast_exp2(mo - mx);
#pragma unroll
        for (int dc = 0; dc < 8; ++dc)
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[dc][i] = fmaf(wa, acc[dc][i], wb * src[dc * 4 + i][lane]);
        l_run = fmaf(wa, l_run, wb * lo);
        m_run = mx;
      }
      __syncthreads();
    }
    if (wave == 0 && r16 < nrows) {
      const size_t slot = (size_t)blockIdx.x + (size_t)b * units + ul;
      float* po = a.sc.part_o + (slot * 16 + r16) * kD;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float4* dst = reinterpret_cast<float4*>(po + 8 * (4 * j4 + i));
        dst[0] = make_float4(acc[0][i], acc[1][i], acc[2][i], acc[3][i]);
        dst[1] = make_float4(acc[4][i], acc[5][i], acc[6][i], acc[7][i]);
      }
      if (j4 == 0) {
        a.sc.part_ml[(slot * 16 + r16) * 2] = m_run;
        a.sc.part_ml[(slot * 16 + r16) * 2 + 1] = l_run;
      }
    }
    r0 += ke - ka;
  }
}

struct FinishMqArgs {
  Shape s;
  LayerView lv;
  Scratch sc;
  void* out;
  SeqMask mask;
  float inv_H;
  int R, Q, HP, passes;
};

constexpr int kFinishThreads = 256;

// Where the attention kernel left the partials of row (head h, query position qi) of sequence b:
// first slot, number of slots, and the row's position inside a slot.
struct RowSpan { size_t slot0; int ns; int row; };
__device__ __forceinline__ RowSpan row_span(const FinishMqArgs& a, int b, int h, int qi, int L) {
  const Shape& s = a.s;
  const int g = h / s.G, hl = h - g * s.G;
  const int pass = hl / a.HP;
  const int ul = g * a.passes + pass;
  const long long off_u = a.sc.offs[b] + (long long)ul * L;
  const long long kf = off_u / a.R, kl = (off_u + L - 1) / a.R;
  RowSpan p;
  p.slot0 = (size_t)kf + (size_t)b * s.Hkv * a.passes + ul;
  p.ns = (int)(kl - kf) + 1;
  p.row = (hl - pass * a.HP) * a.Q + qi;
  return p;
}

// grid (H*Q + ceil(max n_d / 256), B).  Blocks x < H*Q merge the partials of row x = qi*H + h and
// write Att of that query row (Eq. 2).  The other blocks own 256 decode slots each: they rebuild
// the softmax normaliser of every row, and for each slot replay the Q steps in order -- head mean
// of the row's decode-slice probabilities (Eq. 4), then I <- alpha*I + abar (Eq. 5) -- starting
// from I = 0 at the step that appended the slot (Eq. 6); a slot takes no update from query rows
// that precede its own token.
__global__ __launch_bounds__(kFinishThreads) void finish_mq_kernel(const FinishMqArgs a) {
  const Shape& s = a.s;
  const int b = blockIdx.y;
  if (!a.mask.active(b)) return;
  const int Q = a.Q;
  const int M = a.lv.mlen[b];
  const int n1 = a.lv.nd_eff[b];
  const int n0 = n1 - Q;
  const int Lb = M + n1;
  const int rows = s.H * Q;
  const int tid = threadIdx.x, lane = tid & 63;
  constexpr int mlstride = 16 * 2;
  extern __shared__ float smem[];  // row blocks: piece weights; slot blocks: [rows] normalisers + scratch

  if ((int)blockIdx.x < rows) {
    const int qi = blockIdx.x / s.H, h = blockIdx.x - qi * s.H;
    constexpr int SUB = kFinishThreads / kD;
    const int d = tid % kD, sub = tid / kD;
    const RowSpan sp = row_span(a, b, h, qi, Lb);
    const int ns = sp.ns;
    const float* ml = a.sc.part_ml + (sp.slot0 * 16 + sp.row) * 2;
    float mx, L;
    wave_merge_ml(ml, mlstride, ns, lane, mx, L);
    for (int i = tid; i < ns; i += kFinishThreads) smem[i] = fast_exp2(ml[(size_t)i * mlstride] - mx);
    __syncthreads();
    float o0 = 0.f, o1 = 0.f;
    const float* po = a.sc.part_o + (sp.slot0 * 16 + sp.row) * kD + d;
    const size_t ostride = (size_t)16 * kD;
    int i = sub;
    for (; i + SUB < ns; i += 2 * SUB) {
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
      for (int k = 1; k < SUB; ++k) o += red[k * kD + d];
      ((uint16_t*)a.out)[(((size_t)b * Q + qi) * s.H + h) * kD + d] = f32_to_bf16_rne(o / L);
    }
    if (tid == 0) {
      a.sc.lse[((size_t)b * Q + qi) * s.H + h] = mx + log2f(L);
      if (blockIdx.x == 0) {          // the appends become visible to the next kernel
        a.lv.nd[b] = n1;
        a.lv.tpos[b] += Q;
      }
    }
    return;
  }

  const int jb = ((int)blockIdx.x - rows) * kFinishThreads;
  if (jb >= n1) return;
  // normalisers of all rows, `parts` threads per row; smem: [rows], then [parts][rc]
  {
    const int rc = min(rows, kFinishThreads);
    const int parts = kFinishThreads / rc;
    float* red = smem + rows;
    for (int x0 = 0; x0 < rows; x0 += rc) {
      const int xx = tid % rc, part = tid / rc;
      const int x = x0 + xx;
      const bool on = part < parts && x < rows;
      RowSpan sp = {0, 0, 0};
      const float* ml = a.sc.part_ml;
      float m_loc = -INFINITY;
      if (on) {
        const int qi = x / s.H;
        sp = row_span(a, b, x - qi * s.H, qi, Lb);
        ml = a.sc.part_ml + (sp.slot0 * 16 + sp.row) * 2;
        for (int i = part; i < sp.ns; i += parts) m_loc = fmaxf(m_loc, ml[(size_t)i * mlstride]);
        red[part * rc + xx] = m_loc;
      }
      __syncthreads();
      float mx = -INFINITY, l_loc = 0.f;
      if (on) {
        for (int p = 0; p < parts; ++p) mx = fmaxf(mx, red[p * rc + xx]);
        for (int i = part; i < sp.ns; i += parts)
          l_loc = fmaf(fast_exp2(ml[(size_t)i * mlstride] - mx), ml[(size_t)i * mlstride + 1], l_loc);
      }
      __syncthreads();
      if (on) red[part * rc + xx] = l_loc;
      __syncthreads();
      if (on && part == 0) {
        float L = 0.f;
        for (int p = 0; p < parts; ++p) L += red[p * rc + xx];
        smem[x] = mx + log2f(L);   // index qi*H + h
      }
      __syncthreads();
    }
  }
  const int j = jb + tid;
  if (j >= n1) return;
  const size_t si = (size_t)b * s.cap + j;
  float I = (j < n0) ? a.lv.score[si] : 0.f;
  float abar = 0.f;
  // logits of row (h, qi) live at [b][h*Q + qi][slot]
  const float* lg = a.sc.logits + (size_t)b * rows * s.cap + j;
  for (int qi = max(0, j - n0); qi < Q; ++qi) {
    float sum0 = 0.f, sum1 = 0.f;
    const float* lq = lg + (size_t)qi * s.cap;
    const float* nq = smem + qi * s.H;
    const size_t hstride = (size_t)Q * s.cap;
    int h = 0;
    for (; h + 7 < s.H; h += 8) {
      float x[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) x[u] = lq[(size_t)(h + u) * hstride];
#pragma unroll
      for (int u = 0; u < 8; u += 2) {
        sum0 += fast_exp2(x[u] - nq[h + u]);
        sum1 += fast_exp2(x[u + 1] - nq[h + u + 1]);
      }
    }
    for (; h < s.H; ++h) sum0 += fast_exp2(lq[(size_t)h * hstride] - nq[h]);
    abar = (sum0 + sum1) * a.inv_H;
    I = fmaf(s.alpha, I, abar);
  }
  a.lv.score[si] = I;
  a.sc.abar[si] = abar;
}

template <int WPB>
hipError_t launch_mq_w(const MqArgs& a, int n_groups, int* occupancy, hipStream_t st, const KernelTimer* tm) {
  auto kern = attn_mq_kernel<WPB>;
  if (occupancy) return hipOccupancyMaxActiveBlocksPerMultiprocessor(occupancy, kern, WPB * 64, 0);
  if (tm) hipExtLaunchKernelGGL(kern, dim3(n_groups), dim3(WPB * 64), 0, st, tm->start, tm->stop, 0, a);
  else hipLaunchKernelGGL(kern, dim3(n_groups), dim3(WPB * 64), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_mq_v(const MqArgs& a, int n_groups, int* occupancy, hipStream_t st, const KernelTimer* tm) {
  // waves per work-group: variant 1 = 4, default 8
  if (a.s.variant == 1) return launch_mq_w<4>(a, n_groups, occupancy, st, tm);
  return launch_mq_w<8>(a, n_groups, occupancy, st, tm);
}

}  // namespace

int mq_heads_per_pass(int G, int q_len) { return G < 16 / q_len ? G : 16 / q_len; }

hipError_t launch_attn_mq(const Shape& s, const LayerView& lv, const Scratch& sc, int q_len, const void* q,
                          const void* k_new, const void* v_new, const SeqMask& mask, int keys_per_group,
                          int n_groups, hipStream_t st, const KernelTimer* tm) {
  MqArgs a;
  a.s = s; a.lv = lv; a.sc = sc;
  a.q = (const char*)q; a.k_new = (const char*)k_new; a.v_new = (const char*)v_new;
  a.mask = mask; a.R = keys_per_group; a.Q = q_len;
  a.HP = mq_heads_per_pass(s.G, q_len);
  a.passes = (s.G + a.HP - 1) / a.HP;
  return launch_mq_v(a, n_groups, nullptr, st, tm);
}

hipError_t attn_mq_groups_per_cu(const Shape& s, int* out) {
  MqArgs a;
  memset(&a, 0, sizeof a);
  a.s = s;
  return launch_mq_v(a, 0, out, nullptr, nullptr);
}

hipError_t launch_finish_mq(const Shape& s, const LayerView& lv, const Scratch& sc, int q_len, void* out,
                            const SeqMask& mask, int max_nd_eff, int keys_per_group, hipStream_t st,
                            const KernelTimer* tm) {
  FinishMqArgs a;
  a.s = s; a.lv = lv; a.sc = sc; a.out = out; a.mask = mask; a.inv_H = 1.0f / (float)s.H;
  a.R = keys_per_group; a.Q = q_len;
  a.HP = mq_heads_per_pass(s.G, q_len);
  a.passes = (s.G + a.HP - 1) / a.HP;
  const int rows = s.H * q_len;
  dim3 grid(rows + (max_nd_eff + kFinishThreads - 1) / kFinishThreads, s.B);
  const int need = rows + kFinishThreads > s.max_groups ? rows + kFinishThreads : s.max_groups;
  const size_t smem = (size_t)need * sizeof(float);
  if (tm) hipExtLaunchKernelGGL(finish_mq_kernel, grid, dim3(kFinishThreads), smem, st, tm->start, tm->stop, 0, a);
  else hipLaunchKernelGGL(finish_mq_kernel, grid, dim3(kFinishThreads), smem, st, a);
  return hipGetLastError();
}

}  // namespace mkv
