// Decode attention on the matrix cores for bf16 layers with 128-wide heads: the single-query step
// (Q = 1) and the multi-query step (Q <= 16 query rows per sequence and call: chunked or speculative
// decoding, causal among the Q appended tokens).  With the G query heads that share a KV head, a
// pass has up to 16 rows (heads x query positions) against every key -- 32, as two row blocks, when
// G x Q exceeds 16 -- so QK^T and PV are 16-wide contractions and run on MFMA; what is left for
// the vector ALU is the softmax.  Paper: Eq. 2 (attention over the prefill and decode pools),
// Eq. 4-6 (head mean and momentum, applied once per query row in order), Algorithm 1 "append".
//
// gfx950 only: v_mfma_f32_16x16x32_bf16.  Operand layouts (lane l, r = l % 16, j = l / 16):
//   A[m][k] : lane holds m = r, k = 8j .. 8j+7      B[k][n] : lane holds n = r, k = 8j .. 8j+7
//   C[m][n] : lane holds n = r, m = 4j .. 4j+3
#include "mkv_internal.h"
#include "mkv_device.h"

#include <hip/hip_ext.h>

#include <math.h>
#include <string.h>

#include <type_traits>

namespace mkv {
namespace {

using namespace dev;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kD = 128;
constexpr int kRowB = kD * 2;      // bytes per K or V row
constexpr int kNV = kRowB / 16;    // 16-byte vectors per row
constexpr int kTK = 32;            // keys per wave tile
// LDS floats that stage decode logits: real rows x (keys per window).  Every window but a piece's
// last ends in a drain that stops the work-group's stream (stores, their acknowledgement, a barrier).
// Single-query steps: 48 KiB (3072-key windows for the 4 rows of the Llama grouping: one window per
// piece).  Calls with several query rows (BIGWIN): 144 KiB, which the window then shares with the
// buffer through which the waves merge their partial results at the end of a piece -- the two are
// never in use together -- so a 16-row pass gets 2304-key windows and a 32-row pass 1152-key ones
// (it had 768 and 576: four query rows on the ragged Llama layer 72.3 -> 70.3 us, eight rows
// 87.8 -> 83.0 us, sixteen 163 -> 153 us).  The kernel runs one work-group per compute unit anyway
// (registers).
constexpr int kLogitFloats = 12288;
constexpr int kLogitFloatsBig = 36864;

// Decode logits of the matrix-core path, written by the attention kernel and read by the finishing
// kernel: the slot axis is cut into tiles of 64, and a tile holds all rows (head x query position)
// of its 64 slots back to back, [sequence][tile][row][64].  What one finishing wave reads -- every
// row of 64 slots -- is then one contiguous run, not one 256-byte piece per row.
constexpr int kLogitTile = 64;
__device__ __forceinline__ size_t logit_index(const Shape& s, int b, int rows, int row, int slot) {
  const int tiles = (s.cap + kLogitTile - 1) / kLogitTile;
  return (((size_t)b * tiles + slot / kLogitTile) * rows + row) * kLogitTile + slot % kLogitTile;
}

struct MqArgs {
  Shape s;
  LayerView lv;
  Scratch sc;
  const char* q;
  const char* k_new;
  const char* v_new;
  SeqMask mask;
  InlineLens lens;
  int R;        // keys per work-group
  int Q;        // query rows per sequence
  int HP;       // query heads served per pass: min(G, rows per pass / Q)
  int passes;   // passes per KV head: ceil(G / HP)
};

__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4& v) { return __builtin_bit_cast(bf16x8_t, v); }

// c ? x : y on values.  (A conditional between two captured variables is an lvalue, i.e. a choice
// between two addresses followed by a load, which keeps the variables in memory.)
template <typename T>
__device__ __forceinline__ T pick(bool c, T x, T y) { return c ? x : y; }
template <typename T>
__device__ __forceinline__ T pick3(int seg, T x0, T x1, T x2) { return pick(seg == 0, x0, pick(seg == 1, x1, x2)); }

// Untyped buffer descriptor over `bytes` bytes at p: loads past the end return zeros.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, int bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
// 16 bytes at (lane offset + scalar offset) of the buffer
template <int AUX>
__device__ __forceinline__ uint4 buf_load16(rsrc_t r, uint32_t lane_off, uint32_t wave_off) {
  return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, wave_off, AUX));
}

// Same partition of the flattened key axis as the single-query kernel: work-group k takes keys
// [k*R, (k+1)*R), a unit is one KV head x one pass, and every piece of a unit leaves a partial
// (reference, sum, sum p*V) per row in slot  k + unit index.  A unit has L = M + n_d + Q keys.
//
// One wave tile is 32 keys.  Scores: S^T = K * Q^T as two 16-key MFMA tiles, the K rows as the A
// operand (lane (r, j) loads the 16-byte vectors 4*iv + j of key r; the queries are loaded the same
// way, so both operands see the same permutation of the head dimension).  The C layout leaves lane
// (r, j) with the scores of query row r against keys 4j .. 4j+3 of each tile -- which, rounded to
// bf16 (a high and a low part, two MFMAs), is exactly the B operand of  O^T = V^T * P^T  with the
// 32 keys as the contraction index.
// The V^T operand wants, per lane, one head-dim element of 8 keys: lane (r, j) loads vector r of
// the 8 keys it contracts and transposes 16-bit halves in registers (one byte-permute per dword).
// The accumulators then hold O[row r][8 * (4j + i) + dc] for chunk dc, i = 0..3.
//
// NB: row blocks of 16 per pass.  With heads x query positions above 16 a pass carries two blocks
// (32 rows): every K and V tile is then used twice, instead of reading the pool in two passes.
//
// LAZY (deferred compaction, Shape::lazy): decode slots whose token has been evicted still hold
// their rows.  A tile of pool keys comes with the 32 bits of the vector's slot bitmap that cover
// it, and the slot picked by the previous step's selection is compared by value; such keys are
// masked like keys past the end of the segment.  Work-group 0 moves that pending slot into the
// bitmap and clears the half of `pend` that this step's finishing kernel will write.
template <int WPB, int AUXK, int AUXV, int NB, bool LAZY, bool BIGWIN>
__global__ __launch_bounds__(WPB * 64) void attn_mq_kernel(const MqArgs a) {
  constexpr int kRows = 16 * NB;         // rows of a pass = rows of a partial slot
  constexpr int kThreads = WPB * 64;
  const Shape& s = a.s;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);   // tile indices stay scalar
  const int r16 = lane & 15;
  const int j4 = lane >> 4;
  const int Q = a.Q;
  const int units = s.Hkv * a.passes;
  __shared__ long long offs[kMaxBatch + 1];
  constexpr int kWindow = BIGWIN ? kLogitFloatsBig : kLogitFloats;
  // the logit window (rows of SK + 4 floats; the pad spreads the banks) and the merge buffer (every
  // wave's accumulators, reference and sum, lane-major): side by side, or -- BIGWIN -- one buffer
  // with two uses, the window while a piece streams, the merge buffer at its end
  constexpr int kPartFloats = WPB * 34 * 64;
  constexpr int kLogitBuf = kWindow + kRows * 4;
  static_assert(!BIGWIN || kLogitBuf >= kPartFloats, "the merge buffer must fit the logit window");
  __shared__ __align__(16) float sm_logit[kLogitBuf];
  __shared__ float sm_merge[BIGWIN ? 1 : kPartFloats];     // (two arrays: the compiler then knows they are disjoint)
  float (*const sm_part)[34][64] = reinterpret_cast<float (*)[34][64]>(BIGWIN ? sm_logit : sm_merge);
  __shared__ float sm_new[kRows][kTK + 4];   // logits of the appended tokens
  if (wave == 0) build_offsets(s, a.lv, a.mask, units, Q + unit_extra(s), offs, lane, &a.lens);
  else if (wave == 1) warm_kernel_arguments<sizeof(MqArgs)>();   // meanwhile, for all waves of the compute unit
  __syncthreads();
  if (blockIdx.x == 0) {
    for (int b = tid; b <= s.B; b += kThreads) {
      a.sc.offs[b] = offs[b];
      if (b < s.B && a.mask.active(b)) {
        const int nb0 = a.lens.valid ? a.lens.nd[b & (kInlineLens - 1)] : a.lv.nd[b];
        a.lv.nd_eff[b] = nb0 + Q;
        for (int sv = 0; sv < s.S; ++sv) a.sc.evict_key[b * s.S + sv] = ~0ull;   // this step's selection may land here
        if constexpr (LAZY) {
          for (int sv = 0; sv < s.S; ++sv) {
            const int vec = b * s.S + sv;
            const unsigned long long p = a.lv.pend[(size_t)(nb0 & 1) * s.B * s.S + vec];
            if (p != ~0ull) {            // the slot the previous step selected joins the bitmap (once)
              const uint32_t slot = (uint32_t)p;
              uint32_t* w = a.lv.dead + (size_t)vec * s.capw + (slot >> 5);
              const uint32_t old = *w;
              if (!((old >> (slot & 31)) & 1u)) {
                *w = old | (1u << (slot & 31));
                a.lv.nholes[vec] += 1;
              }
            }
            a.lv.pend[(size_t)((nb0 + 1) & 1) * s.B * s.S + vec] = ~0ull;
          }
        }
      }
    }
  }
  const long long total = uniform(offs[s.B]);
  long long r0 = (long long)blockIdx.x * a.R;
  const long long r1 = min(total, r0 + a.R);
  if (r0 >= r1) return;

  int b;
  {
    int lo = 0, hi = s.B;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (uniform(offs[mid]) <= r0) lo = mid; else hi = mid;
    }
    b = uniform(lo);
  }

  while (r0 < r1) {
    while (uniform(offs[b + 1]) <= r0) ++b;
    b = uniform(b);
    const long long ob = uniform(offs[b]);
    const int M = uniform(a.lens.valid ? a.lens.mlen[b & (kInlineLens - 1)] : a.lv.mlen[b]);
    const int n0 = uniform(a.lens.valid ? a.lens.nd[b & (kInlineLens - 1)] : a.lv.nd[b]);
    const int n1 = n0 + Q;
    const int L = M + n1;
    // On the flattened axis a unit is P positions longer than its L keys: the first P positions
    // stand for what starting a piece costs (prologue, merge), so that a work-group whose range
    // crosses a unit boundary gets that many keys fewer.  A range that ends inside them has no keys
    // of the unit and leaves no partial.
    const int Lp = L + unit_extra(s);        // virtual positions in front of the keys and (tail_pad) behind them
    // (a 64-bit division is a long subroutine on the vector ALU; distances below 2^22 take the short way)
    const long long rel = r0 - ob;
    const int ul = uniform(rel < (1 << 22) ? div_small((int)rel, Lp) : (int)(rel / Lp));
    const int g = a.passes == 1 ? ul : uniform(div_small(ul, a.passes));
    const int pass = ul - g * a.passes;
    const int kav = uniform((int)(r0 - ob - (long long)ul * Lp));
    const int kev = uniform((int)min((long long)Lp, kav + (r1 - r0)));
    const int ka = min(max(kav - s.piece_pad, 0), L), ke = min(max(kev - s.piece_pad, 0), L);
    if (ke <= ka) {
      r0 += kev - kav;
      continue;
    }
    const int p0 = min(ka, M), p1 = min(ke, M);
    const int d0 = max(ka, M) - M, d1 = max(ke, M) - M;
    // three kinds of tiles: prefill keys [p0, p1); decode keys that are in the pool already
    // [d0, dp); and appended tokens [a0, d1) of this call, which are still in k_new / v_new
    // (k_new == nullptr: a producer kernel has written the new row into the pool already)
    const bool in_pool = a.k_new == nullptr;
    const int dp = in_pool ? d1 : min(d1, n0);
    const int a0 = max(d0, n0);
    const int ntp = (p1 - p0 + kTK - 1) / kTK;
    const int ntd = (max(dp - d0, 0) + kTK - 1) / kTK;
    const int nta = (!in_pool && d1 > a0) ? 1 : 0;         // Q <= 16 < kTK: one tile holds them
    const int ntile = ntp + ntd + nta;
    const int nrows = min(a.HP, s.G - pass * a.HP) * Q;   // real rows of this pass
    // logit staging window: as many keys as the real rows leave room for (whole tiles)
    const int SK = uniform(div_small(kWindow, nrows)) & ~(kTK - 1);
    const int WT = SK / kTK;
    const int SKP = SK + 4;

    // deferred compaction: the bitmap of the score vector that governs this KV head, and the slot
    // the previous step selected (-1: none)
    [[maybe_unused]] const uint32_t* deadw = nullptr;
    [[maybe_unused]] int pend_slot = -1;
    if constexpr (LAZY) {
      const int vec = b * s.S + (s.S > 1 ? g : 0);
      deadw = a.lv.dead + (size_t)vec * s.capw;
      const unsigned long long p = a.lv.pend[(size_t)(n0 & 1) * s.B * s.S + vec];
      pend_slot = uniform(p == ~0ull ? -1 : (int)(uint32_t)p);
    }
    const size_t head_row = (size_t)uniform(b * s.Hkv + g);
    const char* kpre = (const char*)a.lv.Kp + head_row * (size_t)s.pstride * kRowB;
    const char* vpre = (const char*)a.lv.Vp + head_row * (size_t)s.pstride * kRowB;
    const char* kdec = (const char*)a.lv.Kd + head_row * (size_t)s.dstride * kRowB;
    const char* vdec = (const char*)a.lv.Vd + head_row * (size_t)s.dstride * kRowB;
    // appended token qn of this KV head: row (b, qn, g) of k_new / v_new
    const int new_stride = s.Hkv * kRowB;
    const char* knew = a.k_new + ((size_t)b * Q * s.Hkv + g) * kRowB;
    const char* vnew = a.v_new + ((size_t)b * Q * s.Hkv + g) * kRowB;

    // Append (Alg. 1): the work-group whose piece holds new slots stores their rows for later
    // steps; in this step every reader takes them from k_new / v_new.
    auto append_rows = [&]() __attribute__((always_inline)) {
      if (pass == 0) {
        for (int idx = tid; idx < (in_pool ? 0 : (d1 - a0) * 2 * kNV); idx += kThreads) {
          const int row = idx / (2 * kNV), rem = idx - row * 2 * kNV;
          const int vsel = rem / kNV, vec = rem - vsel * kNV;
          const int jn = a0 + row;
          const char* src = (vsel ? vnew : knew) + (size_t)(jn - n0) * new_stride + vec * 16;
          char* dst = (char*)(vsel ? a.lv.Vd : a.lv.Kd) + (head_row * (size_t)s.dstride + (size_t)jn) * kRowB + vec * 16;
          *reinterpret_cast<uint4*>(dst) = ldg16(src);
        }
        if (g == 0 || s.S > 1) {     // positions: one vector per sequence, or one per KV head
          const int t0 = a.lv.tpos[b];
          const size_t vec = (size_t)b * s.S + (s.S > 1 ? g : 0);
          for (int idx = tid; idx < d1 - a0; idx += kThreads)
            a.lv.pos[vec * s.cap + a0 + idx] = t0 + (a0 + idx - n0);
        }
      }
    };
    // Where it runs: after the first tile has been requested (everything of the piece that waits for
    // memory then arrives in one round trip) -- except with deferred compaction, whose instantiation
    // has no registers to spare for tile registers that live outside the tile loop.
    constexpr bool kEarly = !LAZY;
    if constexpr (!kEarly) append_rows();

    // query rows: row r = (head inside the pass) * Q + (query position); this lane serves rows
    // r16 + 16 * nb
    int qi[NB];
    uint4 qv[NB][4];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int rr = r16 + 16 * nb;
      const int hl = Q == 1 ? rr : div_small(rr, Q);
      qi[nb] = rr - hl * Q;
      const bool row_ok = rr < nrows;
      const char* qp = a.q + (((size_t)b * Q + qi[nb]) * s.H + g * s.G + pass * a.HP + hl) * kRowB;
#pragma unroll
      for (int iv = 0; iv < 4; ++iv) qv[nb][iv] = row_ok ? ldg16(qp + (4 * iv + j4) * 16) : make_uint4(0, 0, 0, 0);
    }
    const int row_base = (g * s.G + pass * a.HP) * Q;      // first row of this pass among the H*Q rows

    float m_run[NB], l_run[NB];             // m_run is identical in the four lanes of a row
    f32x4_t acc[NB][8];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      m_run[nb] = -INFINITY; l_run[nb] = 0.f;
#pragma unroll
      for (int dc = 0; dc < 8; ++dc) acc[nb][dc] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    // K and V come in through buffer loads: a wave-uniform descriptor per segment whose size ends
    // at the segment's last valid row -- rows past it read as zeros, so no lane clamps or branches
    // -- plus one lane offset per operand; the tile's position is a scalar offset.
    //   K: lane (r, j) reads vectors 4*iv + j of row r of each 16-key half
    //   V: lane (r, j) reads vector r of rows 4j + i of each half
    const uint32_t vk_pool = r16 * kRowB + j4 * 16, vv_pool = 4 * j4 * kRowB + r16 * 16;
    const uint32_t vk_new = r16 * new_stride + j4 * 16, vv_new = 4 * j4 * new_stride + r16 * 16;

    // where tile tt starts: segment (0 prefill, 1 pool, 2 appended) and first key of the tile,
    // counted inside the prefill pool or the decode pool
    auto tile_seg = [&](int tt) __attribute__((always_inline)) { return tt < ntp ? 0 : (tt < ntp + ntd ? 1 : 2); };
    auto tile_key = [&](int tt, int seg) __attribute__((always_inline)) {
      return pick3(seg, p0 + tt * kTK, d0 + (tt - ntp) * kTK, a0 + 0);
    };

    const int new_rows = d1 - n0;                           // appended tokens this piece may read
    const int bytes_pre = p1 * kRowB, bytes_dec = max(dp, 0) * kRowB;
    const int bytes_new = new_rows > 0 ? (new_rows - 1) * new_stride + kRowB : 0;

    // Loads of tile tt; a tile index at or past t_end gets an empty descriptor, i.e. zeros and no
    // memory traffic, so that the loop below can always issue its next loads without a branch.
    struct TileAddr { rsrc_t rk, rv; uint32_t vk, vv; int row0, stride; };
    auto tile_addr = [&](int tt, int t_end) __attribute__((always_inline)) {
      const int seg = tile_seg(tt);
      const int jb = tile_key(tt, seg);
      const int bytes = tt < t_end ? pick3(seg, bytes_pre, bytes_dec, bytes_new) : 0;
      TileAddr t;
      t.rk = make_rsrc(pick3(seg, kpre, kdec, knew), bytes);
      t.rv = make_rsrc(pick3(seg, vpre, vdec, vnew), bytes);
      t.stride = pick(seg == 2, new_stride, kRowB);
      t.row0 = pick(seg == 2, jb - n0, jb);                   // first row of the tile in its array
      t.vk = pick(seg == 2, vk_new, vk_pool);
      t.vv = pick(seg == 2, vv_new, vv_pool);
      return t;
    };
    // the two bitmap words that hold the 32 bits of a tile of pool keys (bit i of the tile: key i is
    // an evicted slot); the loads are unconditional like the others (words 0 and 1 for tiles that
    // need none).  The words are cut to the tile's 32 bits only where they are used, a tile later:
    // combined here, the wait for them also held back the next tile's key loads.
    auto load_dead = [&](int tt, int t_end, auto masked) __attribute__((always_inline)) {
      if constexpr (!LAZY || !decltype(masked)::value) return make_uint2(0u, 0u);
      else {
        const int seg = tile_seg(tt);
        const int jb = tile_key(tt, seg);
        const int wi = (seg == 1 && tt < t_end) ? (jb >> 5) : 0;
        return make_uint2(deadw[wi], deadw[wi + 1]);           // the bitmap has two spare words
      }
    };
    auto load_k = [&](int tt, int t_end, uint4 (&kr)[2][4]) __attribute__((always_inline)) {
      const TileAddr t = tile_addr(tt, t_end);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint32_t so = (uint32_t)(t.row0 + 16 * h) * (uint32_t)t.stride;
#pragma unroll
        for (int iv = 0; iv < 4; ++iv) kr[h][iv] = buf_load16<AUXK>(t.rk, t.vk + iv * 64, so);
      }
    };
    auto load_v = [&](int tt, int t_end, uint4 (&vr)[2][4]) __attribute__((always_inline)) {
      const TileAddr t = tile_addr(tt, t_end);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint32_t so = (uint32_t)(t.row0 + 16 * h) * (uint32_t)t.stride;
#pragma unroll
        for (int i = 0; i < 4; ++i) vr[h][i] = buf_load16<AUXV>(t.rv, t.vv, so + (uint32_t)(i * t.stride));
      }
    };

    int win = 0;
    constexpr float kSlack = 8.0f;
    // scores of one tile against the rows of each block: x[nb][4h + i] = logit of key 16h + 4j + i (base 2), -inf
    // where masked; decode logits are staged for the score update
    auto score_tile = [&](int tt, const uint4 (&kr)[2][4], uint2 dwords, auto masked, float (&x)[NB][8]) __attribute__((always_inline)) {
      const int seg = tile_seg(tt);
      const int jb = tile_key(tt, seg);
      [[maybe_unused]] const uint32_t dmask = __builtin_amdgcn_alignbit(dwords.y, dwords.x, (uint32_t)jb & 31u);
      const int jn = pick3(seg, p1, dp, d1);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int rr = r16 + 16 * nb;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          f32x4_t sv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int iv = 0; iv < 4; ++iv)
            sv = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kr[h][iv]), as_bf16x8(qv[nb][iv]), sv, 0, 0, 0);
          const int key0 = jb + 16 * h + 4 * j4;
          float4 st;
          st.x = sv[0] * s.scale_log2; st.y = sv[1] * s.scale_log2;
          st.z = sv[2] * s.scale_log2; st.w = sv[3] * s.scale_log2;
          if (seg == 1 && rr < nrows) *reinterpret_cast<float4*>(&sm_logit[rr * SKP + (tt - ntp - win * WT) * kTK + 16 * h + 4 * j4]) = st;
          if (seg == 2) *reinterpret_cast<float4*>(&sm_new[rr][16 * h + 4 * j4]) = st;
          const float sx[4] = {st.x, st.y, st.z, st.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int key = key0 + i;
            // past the segment, or an appended token that comes after this row's own (causal order)
            bool ok = key < jn && !(seg == 2 && key - n0 > qi[nb]);
            if constexpr (LAZY && decltype(masked)::value)      // an evicted slot that still holds its rows
              ok = ok && !(seg == 1 && (((dmask >> (16 * h + 4 * j4 + i)) & 1u) || key == pend_slot));
            x[nb][4 * h + i] = ok ? sx[i] : -INFINITY;
          }
        }
      }
    };
    struct PairB { bf16x8_t hi, lo; };
    // running softmax over the tile's scores; returns the probabilities as bf16 B operands
    auto softmax_tile = [&](const float (&x)[8], float& m_r, float& l_r, f32x4_t (&ac)[8]) __attribute__((always_inline)) {
      float tm = x[0];
#pragma unroll
      for (int i = 1; i < 8; ++i) tm = fmaxf(tm, x[i]);
      if (__any(tm > m_r + kSlack)) {
        // the four lanes of a row raise the reference together, to the row's maximum over the tile
        tm = fmaxf(tm, __shfl_xor(tm, 16));
        tm = fmaxf(tm, __shfl_xor(tm, 32));
        if (tm > m_r + kSlack) {
          const float cf = fast_exp2(m_r - tm);   // exp2(-inf) = 0 on the first raise
          l_r *= cf;
          m_r = tm;
#pragma unroll
          for (int dc = 0; dc < 8; ++dc) ac[dc] *= cf;
        }
      }
      // the probability enters the value contraction as two bf16 terms, p = hi + lo up to 2^-17:
      // with hi alone (2^-9) an output over a handful of keys can miss the bf16 tolerance
      PairB pb;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float p = (x[i] == -INFINITY) ? 0.f : fast_exp2(x[i] - m_r);
        l_r += p;
        const __bf16 hi = (__bf16)p;
        pb.hi[i] = hi;
        pb.lo[i] = (__bf16)(p - (float)hi);
      }
      return pb;
    };
    // acc += V^T P^T.  V^T operand for chunk dc: element 4h + i = bf16 number dc of the vector of
    // key 4j + i, half h
    auto value_tile = [&](const uint4 (&vr)[2][4], const PairB (&pb)[NB]) __attribute__((always_inline)) {
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
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          acc[nb][dc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(av), pb[nb].hi, acc[nb][dc], 0, 0, 0);
          acc[nb][dc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(av), pb[nb].lo, acc[nb][dc], 0, 0, 0);
        }
      }
    };

    // Tiles [t_lo, t_hi), round-robin over the waves, as a two-stage pipeline on one set of
    // registers: as soon as the scores of a tile are formed its K registers take the next tile's
    // K, and as soon as the values are accumulated its V registers take the next tile's V, so a
    // wave always has loads in flight.
    // `masked`: the piece holds keys of the decode pool, whose slots may be marked (LAZY only); a
    // piece of prompt keys alone runs the plain loop
    // requests a wave's first tile of [t_lo, t_hi); returns the tile's bitmap bits
    auto prime = [&](int t_lo, int t_hi, auto masked, uint4 (&kbuf)[2][4], uint4 (&vbuf)[2][4]) __attribute__((always_inline)) {
      const int tt = t_lo + wave;
      const uint2 bits = load_dead(tt, t_hi, masked);
      load_k(tt, t_hi, kbuf);
      load_v(tt, t_hi, vbuf);
      return bits;
    };
    auto tile_loop = [&](int t_lo, int t_hi, auto masked, uint2 dmask, uint4 (&kbuf)[2][4], uint4 (&vbuf)[2][4]) __attribute__((always_inline)) {
      int tt = t_lo + wave;
      while (tt < t_hi) {
        float x[NB][8];
        score_tile(tt, kbuf, dmask, masked, x);
        dmask = load_dead(tt + WPB, t_hi, masked);
        load_k(tt + WPB, t_hi, kbuf);
        PairB pb[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) pb[nb] = softmax_tile(x[nb], m_run[nb], l_run[nb], acc[nb]);
        value_tile(vbuf, pb);
        load_v(tt + WPB, t_hi, vbuf);
        tt += WPB;
      }
    };
    // kEarly: the tile registers live at piece scope, and the first window's first tile (`primed`)
    // is already under way when its loop starts
    [[maybe_unused]] uint4 kbuf0[2][4], vbuf0[2][4];
    auto run_tiles = [&](int t_lo, int t_hi, auto masked, [[maybe_unused]] bool primed) __attribute__((always_inline)) {
      if constexpr (kEarly) {
        uint2 dmask = make_uint2(0u, 0u);
        if (!primed) dmask = prime(t_lo, t_hi, masked, kbuf0, vbuf0);
        tile_loop(t_lo, t_hi, masked, dmask, kbuf0, vbuf0);
      } else {
        uint4 kbuf[2][4], vbuf[2][4];
        const uint2 dmask = prime(t_lo, t_hi, masked, kbuf, vbuf);
        tile_loop(t_lo, t_hi, masked, dmask, kbuf, vbuf);
      }
    };

    // phases: all prefill tiles plus the first window of pool tiles, then one window per phase (the
    // tile of appended tokens rides with the last); the staged logits of a window are written out
    // by the whole work-group
    if constexpr (kEarly) (void)prime(0, min(ntile, ntp + WT), std::false_type{}, kbuf0, vbuf0);
    if constexpr (kEarly) append_rows();
    for (int t_lo = 0; t_lo < ntile; ++win) {
      const int t_hi = min(ntile, ntp + (win + 1) * WT);
      if (LAZY && ntd > 0) run_tiles(t_lo, t_hi, std::true_type{}, false);
      else run_tiles(t_lo, t_hi, std::false_type{}, kEarly && (BIGWIN || t_lo == 0));   // BIGWIN: every window finds its first tile requested
      const int wk0 = win * SK;
      const int nk = min(dp - d0 - wk0, SK);
      const bool last = t_hi == ntile;
      if (nk > 0 || (last && nta)) {
        __syncthreads();
        if (nk > 0) {
          // the window's slots [s_lo, s_hi) go out four at a time: an item is (row, quad of slots
          // 4k .. 4k+3), one 16-byte store (a quad never straddles a 64-slot tile of the logit
          // layout); the quads at the window's ends may be partial and go out float by float
          const int s_lo = d0 + wk0, s_hi = s_lo + nk;
          const int q_lo = s_lo & ~3;
          const int nq = (s_hi - q_lo + 3) >> 2;
          const bool aligned = (s_lo & 3) == 0;            // then the LDS side is 16-byte aligned as well
          for (int item = tid; item < nrows * nq; item += kThreads) {
            const int r = div_small(item, nq);
            const int sq = q_lo + 4 * (item - r * nq);
            float* dst = a.sc.logits + logit_index(s, b, s.H * Q, row_base + r, sq);
            const float* src = sm_logit + r * SKP + (sq - s_lo);
            if (sq >= s_lo && sq + 4 <= s_hi) {
              float4 v;
              if (aligned) v = *reinterpret_cast<const float4*>(src);
              else v = make_float4(src[0], src[1], src[2], src[3]);
              *reinterpret_cast<float4*>(dst) = v;
            } else {
#pragma unroll
              for (int i = 0; i < 4; ++i)
                if (sq + i >= s_lo && sq + i < s_hi) dst[i] = src[i];
            }
          }
        }
        if (last && nta) {
          const int nn = d1 - a0;
          for (int idx = tid; idx < nrows * nn; idx += kThreads) {
            const int r = idx / nn, key = idx - r * nn;
            a.sc.logits[logit_index(s, b, s.H * Q, row_base + r, a0 + key)] = sm_new[r][key];
          }
        }
        if (!last) {
          // the next window's first tile is requested behind the stores: the wait for the stores
          // (loads and stores share the completion counter) then covers its round trip as well
          if constexpr (kEarly && BIGWIN) (void)prime(t_hi, min(ntile, ntp + (win + 2) * WT), std::false_type{}, kbuf0, vbuf0);
          __builtin_amdgcn_s_waitcnt(0x0F70);
          __syncthreads();
        }
      }
      t_lo = t_hi;
    }
    // waves -> one partial per piece, a block of 16 rows at a time: every wave leaves its
    // accumulators, reference and sum in LDS (lane-major, conflict-free); after one barrier, thread
    // (lane, i, q) merges four consecutive output elements over the waves and stores them.
    // (BIGWIN: the merge buffer is the logit window; a piece with decode keys has just written its
    // last window out, and every wave must have read its share before the buffer is overwritten.)
    if constexpr (BIGWIN) {
      if (ntd + nta > 0) __syncthreads();
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      // the four lanes of a row saw different keys: add up their sums (the accumulators are
      // already contracted over all keys of the wave)
      float l_row = l_run[nb];
      l_row += __shfl_xor(l_row, 16);
      l_row += __shfl_xor(l_row, 32);
      if (nb > 0) __syncthreads();       // sm_part still holds the previous block
      {
        float (*dst)[64] = sm_part[wave];
#pragma unroll
        for (int dc = 0; dc < 8; ++dc)
#pragma unroll
          for (int i = 0; i < 4; ++i) dst[dc * 4 + i][lane] = acc[nb][dc][i];
        dst[32][lane] = m_run[nb];
        dst[33][lane] = l_row;
      }
      __syncthreads();
      for (int item = tid; item < 64 * 8; item += kThreads) {
        const int ln = item & 63, iq = item >> 6;       // source lane; (i, q) = (iq & 3, iq >> 2)
        const int row = (ln & 15) + 16 * nb, jj = ln >> 4, i = iq & 3, q = iq >> 2;
        if (row < nrows) {
          float mx = sm_part[0][32][ln];
#pragma unroll
          for (int w = 1; w < WPB; ++w) mx = fmaxf(mx, sm_part[w][32][ln]);
          float o[4] = {0.f, 0.f, 0.f, 0.f}, lt = 0.f;
#pragma unroll
          for (int w = 0; w < WPB; ++w) {
            const float mw = sm_part[w][32][ln];
            // a wave without visible keys has reference -inf; if no wave had any, mx is -inf as well
            const float e = (mw == -INFINITY) ? 0.f : fast_exp2(mw - mx);
            lt = fmaf(e, sm_part[w][33][ln], lt);
#pragma unroll
            for (int c = 0; c < 4; ++c) o[c] = fmaf(e, sm_part[w][(4 * q + c) * 4 + i][ln], o[c]);
          }
          const size_t slot = (size_t)blockIdx.x + (size_t)b * units + ul;
          // accumulator (dc, i) of lane (row, jj) is output element 8 * (4 jj + i) + dc
          *reinterpret_cast<float4*>(a.sc.part_o + (slot * kRows + row) * kD + 8 * (4 * jj + i) + 4 * q) =
              make_float4(o[0], o[1], o[2], o[3]);
          if (jj == 0 && iq == 0) {
            a.sc.part_ml[(slot * kRows + row) * 2] = mx;
            a.sc.part_ml[(slot * kRows + row) * 2 + 1] = lt;
          }
        }
      }
    }
    __syncthreads();   // sm_part is reused by the next piece
    r0 += kev - kav;
  }
}

struct FinishMqArgs {
  Shape s;
  LayerView lv;
  Scratch sc;
  void* out;
  SeqMask mask;
  InlineLens lens;
  float inv_H;
  int R, Q, HP, passes;
  int RPS;      // rows per partial slot: 16 x row blocks of the attention pass
  int narrow;   // the flattened key axis of the launch fits 31 bits: slot arithmetic in 32-bit divisions
};

constexpr int kFinishThreads = 256;
constexpr int kSlotsMulti = 64;       // decode slots per slot block when a call has several query rows
constexpr int kRowsPerBlock = kFinishThreads / 64;   // output rows merged per work-group: one per wave

// Where the attention kernel left the partials of row (head h, query position qi) of sequence b:
// first slot, number of slots, and the row's position inside a slot.
struct RowSpan { size_t slot0; int ns; int row; };
__device__ __forceinline__ RowSpan row_span(const FinishMqArgs& a, long long off_b, int b, int h, int qi, int L) {
  const Shape& s = a.s;
  const int g = h / s.G, hl = h - g * s.G;
  const int pass = hl / a.HP;
  const int ul = g * a.passes + pass;
  const long long off_u = off_b + (long long)ul * (L + unit_extra(s)) + s.piece_pad;   // the unit's first key on the flattened axis
  long long kf, kl;
  if (a.narrow) {       // (a 64-bit division is a long subroutine, and the loads below wait for it)
    kf = (uint32_t)off_u / (uint32_t)a.R;
    kl = (uint32_t)(off_u + L - 1) / (uint32_t)a.R;
  } else {
    kf = off_u / a.R;
    kl = (off_u + L - 1) / a.R;
  }
  RowSpan p;
  p.slot0 = (size_t)kf + (size_t)b * s.Hkv * a.passes + ul;
  p.ns = (int)(kl - kf) + 1;
  p.row = (hl - pass * a.HP) * a.Q + qi;
  return p;
}

// grid (ceil(H*Q / 4) + ceil(max n_d / slots per block), B).  The first blocks merge the partials of
// four rows x = qi*H + h each, one wave per row, and write Att of those query rows (Eq. 2).  The other
// blocks own 256 (single-row instantiation) or 64 decode slots each: they rebuild
// the softmax normaliser of every row, and for each slot replay the Q steps in order -- head mean
// of the row's decode-slice probabilities (Eq. 4), then I <- alpha*I + abar (Eq. 5) -- starting
// from I = 0 at the step that appended the slot (Eq. 6); a slot takes no update from query rows
// that precede its own token.
//
// ONE: a single query row and at most 32 heads (the plain decode step of the usual layers), where a
// slot's logits fit in registers and are fetched before the normalisers are rebuilt.
// LAZY: deferred compaction (Shape::lazy); a separate instantiation so that the ordinary one
// carries none of its loads and tests.
template <bool ONE, bool LAZY>
__global__ __launch_bounds__(kFinishThreads) void finish_mq_kernel(const FinishMqArgs a) {
  warm_kernel_arguments<sizeof(FinishMqArgs)>();
  const Shape& s = a.s;
  const int b = blockIdx.y;
  if (!a.mask.active(b)) return;
  const int Q = ONE ? 1 : a.Q;
  // lengths and the sequence's start on the flattened key axis: with the launch arguments when the
  // batch is small (no memory round trip before the first useful load), else from memory
  const bool il = a.lens.valid;
  const int M = il ? a.lens.mlen[b & (kInlineLens - 1)] : a.lv.mlen[b];
  const int n1 = il ? a.lens.nd[b & (kInlineLens - 1)] + Q : a.lv.nd_eff[b];
  const long long off_b = il ? a.lens.offs[b & (kInlineLens - 1)] : a.sc.offs[b];
  const int n0 = n1 - Q;
  const int Lb = M + n1;
  const int rows = s.H * Q;
  const int tid = threadIdx.x, lane = tid & 63;
  const int mlstride = a.RPS * 2;
  extern __shared__ float smem[];  // slot blocks: [rows] normalisers + exchange space

  const int row_blocks = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
  // Order of the blocks along x.  ONE: row blocks first (everything is resident at once).  Otherwise
  // the slot blocks come first: a launch has more blocks than the chip holds, the slot blocks are
  // the long ones (two dependent round trips), and blocks start in index order.
  const int slot_blocks = (int)gridDim.x - row_blocks;
  const int rblk = ONE ? (int)blockIdx.x : (int)blockIdx.x - slot_blocks;
  const int sblk = ONE ? (int)blockIdx.x - row_blocks : (int)blockIdx.x;
  if (rblk >= 0 && rblk < row_blocks) {
    // one wave per row, a lane per pair of output elements: no LDS, no barrier
    const int x = rblk * kRowsPerBlock + (tid >> 6);
    if (x >= rows) return;
    const int qi = x / s.H, h = x - qi * s.H;
    const RowSpan sp = row_span(a, off_b, b, h, qi, Lb);
    const int ns = sp.ns;
    const float* ml = a.sc.part_ml + (sp.slot0 * a.RPS + sp.row) * 2;
    const float2* po = reinterpret_cast<const float2*>(a.sc.part_o + (sp.slot0 * a.RPS + sp.row) * kD) + lane;
    const size_t ostride = (size_t)a.RPS * kD / 2;
    // the first pieces' partial outputs are fetched alongside the (reference, sum) pairs rather
    // than after the weights are known: sixteen covers every row of a batch that fills the chip,
    // and half the pieces of a single sequence spread over all work-groups (with four up front and
    // eight per further round the batch-1 Llama layer took 16.2 us per step, now 15.8)
    constexpr int kPrePieces = 16;
    float2 pre[kPrePieces];
#pragma unroll
    // (every load unconditional -- a piece index past the end re-reads the last piece and gets no
    // weight below: a predicate per load is a branch out of line and back per load)
    for (int i = 0; i < kPrePieces; ++i) pre[i] = po[(size_t)min(i, ns - 1) * ostride];
    float mx, L, m_first;                // m_first: reference of piece `lane`
    wave_merge_ml(ml, mlstride, ns, lane, mx, L, &m_first);
    float2 o = make_float2(0.f, 0.f);
#pragma unroll
    for (int i = 0; i < kPrePieces; ++i) {
      const float w = fast_exp2(__shfl(m_first, i) - mx);     // 0 for a piece without visible keys
      if (i < ns) { o.x = fmaf(w, pre[i].x, o.x); o.y = fmaf(w, pre[i].y, o.y); }
    }
    // further pieces (few sequences spread over many work-groups), sixteen loads at a time
    for (int i0 = kPrePieces; i0 < ns; i0 += 16) {
      float2 v[16];
      float w[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const int i = min(i0 + k, ns - 1);
        v[k] = po[(size_t)i * ostride];
        w[k] = ml[(size_t)i * mlstride];
      }
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const float e = i0 + k < ns ? fast_exp2(w[k] - mx) : 0.f;
        o.x = fmaf(e, v[k].x, o.x); o.y = fmaf(e, v[k].y, o.y);
      }
    }
    const uint32_t packed = (uint32_t)f32_to_bf16_rne(o.x / L) | ((uint32_t)f32_to_bf16_rne(o.y / L) << 16);
    reinterpret_cast<uint32_t*>(a.out)[((((size_t)b * Q + qi) * s.H + h) * kD) / 2 + lane] = packed;
    if (lane == 0) {
      a.sc.lse[((size_t)b * Q + qi) * s.H + h] = mx + log2f(L);
      if (x == 0) {                   // the appends become visible to the next kernel
        a.lv.nd[b] = n1;
        a.lv.tpos[b] += Q;
      }
    }
    return;
  }

  // slots per slot block: a thread per slot (ONE), or a lane per slot with the query rows dealt out
  // to the four waves
  constexpr int kSlots = ONE ? kFinishThreads : kSlotsMulti;
  const int jb = sblk * kSlots;
  if (jb >= n1) return;
  const int j = jb + (ONE ? tid : lane);
  // ONE: the slot's logits are fetched before the normalisers are rebuilt, so that the two memory
  // round trips overlap
  constexpr int kPre = ONE ? 32 : 1;
  float xpre[kPre];
  constexpr int kPreS = 8;               // score vectors whose previous value is fetched up front too
  float ipre[kPreS];
  // deferred compaction: the word of the vector's slot bitmap that holds this slot's bit
  // and its hole count, which decides whether this step selects (first vector up front, the
  // usual single one; further vectors fetch theirs when their turn comes)
  [[maybe_unused]] uint32_t dpre0 = 0u;
  [[maybe_unused]] int hpre0 = 0;
  if constexpr (LAZY) {
    if (j < n1) dpre0 = a.lv.dead[(size_t)b * s.S * s.capw + (j >> 5)];
    hpre0 = a.lv.nholes[b * s.S];
  }
  if (j < n1) {
    if constexpr (ONE) {
      const float* lg0 = a.sc.logits + logit_index(s, b, rows, 0, j);
#pragma unroll
      // (unconditional as well; heads past H - 1 repeat the last head and are never summed)
      for (int h = 0; h < kPre; ++h) xpre[h] = lg0[min(h, s.H - 1) * kLogitTile];
    }
    ipre[0] = j < n0 ? a.lv.score[(size_t)b * s.S * s.cap + j] : 0.f;
#pragma unroll
    for (int sv = 1; sv < kPreS; ++sv) ipre[sv] = 0.f;
    if (s.S > 1) {       // one vector per KV head: their previous values too
#pragma unroll
      for (int sv = 1; sv < kPreS; ++sv)
        ipre[sv] = (sv < s.S && j < n0) ? a.lv.score[((size_t)b * s.S + sv) * s.cap + j] : 0.f;
    }
  }
  // ONE: every wave rebuilds the (at most 32) normalisers by itself, in registers: lane l takes
  // row l % 32 and the pieces of parity l / 32, the two halves meet through one lane exchange, and
  // the sums below read row h's value from lane h -- no LDS, no barrier.
  [[maybe_unused]] float lse_lane = 0.f;
  if constexpr (ONE) {
    const int x = lane & 31, half = lane >> 5;
    float m_loc = -INFINITY, l_loc = 0.f;
    if (x < rows) {
      const RowSpan sp = row_span(a, off_b, b, x, 0, Lb);
      const float2* ml = reinterpret_cast<const float2*>(a.sc.part_ml) + (sp.slot0 * a.RPS + sp.row);
      for (int i0 = half; i0 < sp.ns; i0 += 16) {    // eight loads in flight (sixteen: 0.3 us faster with 32
        float2 v[8];                                 // pieces per row, 0.3 us slower with the usual two or three)
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = ml[(size_t)min(i0 + 2 * k, sp.ns - 1) * a.RPS];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          if (i0 + 2 * k >= sp.ns) continue;
          if (v[k].x > m_loc) {            // a piece without visible keys has reference -inf, sum 0
            l_loc = fmaf(l_loc, fast_exp2(m_loc - v[k].x), v[k].y);
            m_loc = v[k].x;
          } else if (v[k].x != -INFINITY) {
            l_loc = fmaf(v[k].y, fast_exp2(v[k].x - m_loc), l_loc);
          }
        }
      }
    }
    const float m_o = __shfl_xor(m_loc, 32), l_o = __shfl_xor(l_loc, 32);
    const float mx = fmaxf(m_loc, m_o);
    float L = 0.f;
    if (m_loc != -INFINITY) L = l_loc * fast_exp2(m_loc - mx);
    if (m_o != -INFINITY) L = fmaf(l_o, fast_exp2(m_o - mx), L);
    lse_lane = mx + log2f(L);
  }
  // otherwise: normalisers of all rows, `parts` threads per row, each folding its share of the row's pieces
  // into a running (reference, sum) pair from one round of loads; smem: [rows], then two arrays
  // [parts][rc] through which the parts of a row meet
  if constexpr (!ONE) {
    const int rc = min(rows, kFinishThreads);
    const int parts = kFinishThreads / rc;
    float* red_m = smem + rows;
    float* red_l = red_m + kFinishThreads;
    for (int x0 = 0; x0 < rows; x0 += rc) {
      const int xx = tid % rc, part = tid / rc;
      const int x = x0 + xx;
      const bool on = part < parts && x < rows;
      if (on) {
        const int qi = x / s.H;
        const RowSpan sp = row_span(a, off_b, b, x - qi * s.H, qi, Lb);
        const float2* ml = reinterpret_cast<const float2*>(a.sc.part_ml) + (sp.slot0 * a.RPS + sp.row);
        float m_loc = -INFINITY, l_loc = 0.f;
        for (int i0 = part; i0 < sp.ns; i0 += 4 * parts) {   // four loads in flight
          float2 v[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) v[k] = ml[(size_t)min(i0 + k * parts, sp.ns - 1) * a.RPS];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            if (i0 + k * parts >= sp.ns) continue;
            if (v[k].x > m_loc) {          // a piece without visible keys has reference -inf, sum 0
              l_loc = fmaf(l_loc, fast_exp2(m_loc - v[k].x), v[k].y);
              m_loc = v[k].x;
            } else if (v[k].x != -INFINITY) {
              l_loc = fmaf(v[k].y, fast_exp2(v[k].x - m_loc), l_loc);
            }
          }
        }
        red_m[part * rc + xx] = m_loc;
        red_l[part * rc + xx] = l_loc;
      }
      __syncthreads();
      if (on && part == 0) {
        float mx = -INFINITY;
        for (int p = 0; p < parts; ++p) mx = fmaxf(mx, red_m[p * rc + xx]);
        float L = 0.f;
        for (int p = 0; p < parts; ++p) {
          const float mp = red_m[p * rc + xx];
          if (mp != -INFINITY) L = fmaf(red_l[p * rc + xx], fast_exp2(mp - mx), L);
        }
        smem[x] = mx + log2f(L);   // index qi*H + h
      }
      __syncthreads();
    }
  }
  // One token appended and exactly one to evict (trigger = budget, pool at budget + 1 live
  // tokens): the selection of Eq. 8 is an arg-min over the scores computed right here; every slot
  // block merges its candidates' minimum into the vector's selection key -- evict_key for the row
  // shift that follows, or, with deferred compaction, the half of `pend` that belongs to a pool of
  // n1 slots.
  const bool one_out = Q == 1 && s.trigger == s.budget;
  // One score vector per sequence (mean over all H heads, Eq. 4 as printed) or one per KV head
  // (mean over the G heads of the group): vector sv covers heads [sv*Hs, (sv+1)*Hs).
  const int Hs = s.H / s.S;
  const float inv_Hs = 1.0f / (float)Hs;
  __shared__ unsigned long long key_slots[4];
  [[maybe_unused]] __shared__ float sm_abar[ONE ? 1 : 16][kSlotsMulti];   // head means per (query row, slot)
#pragma unroll 1
  for (int sv = 0; sv < s.S; ++sv) {
    unsigned long long key = ~0ull;
    const size_t si = ((size_t)b * s.S + sv) * s.cap + j;
    const int vec = b * s.S + sv;
    int holes = 0;
    uint32_t dword = 0u;
    if constexpr (LAZY) {
      if (sv == 0) {
        holes = hpre0;
        dword = dpre0;
      } else {
        holes = a.lv.nholes[vec];
        if (j < n1) dword = a.lv.dead[(size_t)vec * s.capw + (j >> 5)];
      }
    }
    const bool pick_one = one_out && n1 - holes == s.budget + 1;
    unsigned long long* key_dst = LAZY ? a.lv.pend + (size_t)(n1 & 1) * s.B * s.S + vec : a.sc.evict_key + vec;
    float I = 0.f;                       // previous score of the slot (0 for one appended now, Eq. 6)
    if (sv < kPreS) {
      I = ipre[0];
#pragma unroll
      for (int u = 1; u < kPreS; ++u) I = (sv == u) ? ipre[u] : I;
    } else if (j < n0) {
      I = a.lv.score[si];
    }
    const bool alive = !LAZY || !((dword >> (j & 31)) & 1u);   // an evicted slot takes no update and is no candidate
    if constexpr (ONE) {
      if (j < n1) {
        float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
        for (int h = 0; h < kPre; h += 2) {
          const float n0h = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lse_lane), h));
          const float n1h = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lse_lane), h + 1));
          if (h >= sv * Hs && h < (sv + 1) * Hs) sum0 += fast_exp2(xpre[h] - n0h);
          if (h + 1 >= sv * Hs && h + 1 < (sv + 1) * Hs) sum1 += fast_exp2(xpre[h + 1] - n1h);
        }
        const float abar = alive ? (sum0 + sum1) * inv_Hs : 0.f;
        I = fmaf(s.alpha, I, abar);
        if (alive) a.lv.score[si] = I;
        a.sc.abar[si] = abar;
        if (pick_one && alive && j < n1 - s.window) key = evict_key_of(I, j);
      }
    } else {
      // Head means first, the recurrence after: wave w forms abar of query rows w, w+4, ... for
      // its 64 slots (independent of each other, so the rows of a call are in flight together),
      // then wave 0 applies Eq. 5 row by row.  Logits of row (h, qi) are row h*Q + qi of the slot's tile;
      // a wave walks its (row, 32 heads) chunks one chunk ahead of the arithmetic, the same walk
      // in every lane (heads clamped to the last one).
      const int w = tid >> 6;
      if (j < n1) {
        constexpr int CH = 32;
        const float* lg = a.sc.logits + logit_index(s, b, rows, sv * Hs * Q, j);
        const int hstride = Q * kLogitTile;
        const int nch = (Hs + CH - 1) / CH;
        float xa[CH], xb[CH];
        int qi = w, c = 0;                // wave-uniform
        auto fetch = [&](int qf, int cf, float (&x)[CH]) __attribute__((always_inline)) {
          const float* src = lg + qf * kLogitTile;
#pragma unroll
          for (int u = 0; u < CH; ++u) x[u] = src[min(cf * CH + u, Hs - 1) * hstride];
        };
        if (qi < Q) fetch(qi, 0, xa);
        float sum0 = 0.f, sum1 = 0.f;
        // one chunk: request the next one into `nxt`, then consume `cur` (nothing past the last row)
        auto stage = [&](const float (&cur)[CH], float (&nxt)[CH]) __attribute__((always_inline)) {
          if (qi >= Q) return;
          int qn = qi, cn = c + 1;
          if (cn == nch) { cn = 0; qn = qi + kFinishThreads / 64; }
          if (qn < Q) fetch(qn, cn, nxt);
          const float* nq = smem + qi * s.H + sv * Hs + c * CH;
#pragma unroll
          for (int u = 0; u < CH; u += 2) {
            if (c * CH + u < Hs) sum0 += fast_exp2(cur[u] - nq[u]);
            if (c * CH + u + 1 < Hs) sum1 += fast_exp2(cur[u + 1] - nq[u + 1]);
          }
          if (cn == 0) {                 // the row is complete: Eq. 4
            sm_abar[qi][lane] = (sum0 + sum1) * inv_Hs;
            sum0 = sum1 = 0.f;
          }
          qi = qn; c = cn;
        };
        while (qi < Q) {                 // the two register sets swap roles: no copies, no early waits
          stage(xa, xb);
          stage(xb, xa);
        }
      }
      __syncthreads();
      if (w == 0 && j < n1) {
        // a slot appended by this call takes no update from the rows before its own token
        float abar = 0.f;
        for (int qi = max(0, j - n0); qi < Q; ++qi) {
          abar = sm_abar[qi][lane];
          I = fmaf(s.alpha, I, abar);    // Eq. 5
        }
        if (alive) a.lv.score[si] = I;
        a.sc.abar[si] = alive ? abar : 0.f;
        if (pick_one && alive && j < n1 - s.window) key = evict_key_of(I, j);
      }
      if (sv + 1 < s.S) __syncthreads();   // the next vector reuses sm_abar
    }
    if (pick_one) block_min_key_to(key, key_dst, key_slots, tid);
  }
}

template <int WPB, int AUXK = 0, int AUXV = 0, int NB = 1, bool LAZY = false, bool BIGWIN = false>
hipError_t launch_mq_w(const MqArgs& a, int n_groups, int* occupancy, hipStream_t st, const KernelTimer* tm) {
  auto kern = attn_mq_kernel<WPB, AUXK, AUXV, NB, LAZY, BIGWIN>;
  if (occupancy) return hipOccupancyMaxActiveBlocksPerMultiprocessor(occupancy, kern, WPB * 64, 0);
  if (tm) hipExtLaunchKernelGGL(kern, dim3(n_groups), dim3(WPB * 64), 0, st, tm->start, tm->stop, 0, a);
  else hipLaunchKernelGGL(kern, dim3(n_groups), dim3(WPB * 64), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_mq_v(const MqArgs& a, int n_groups, int* occupancy, hipStream_t st, const KernelTimer* tm) {
  // more than 16 rows (heads x query positions): two row blocks per pass
  if (mq_row_blocks(a.s.G, a.Q) == 2) return launch_mq_w<8, 0, 2, 2, false, true>(a, n_groups, occupancy, st, tm);
  // several query rows in one row block, or a decode pool that the small window cannot hold in one
  // go (every further window costs the work-group a drain in mid-stream): the large logit window
  // (default variant only)
  const int rows_most = (a.s.G < a.HP ? a.s.G : a.HP) * a.Q;
  if ((a.Q > 1 || (long long)a.s.cap * rows_most > kLogitFloats) && a.s.variant == 0 && !a.s.lazy)
    return launch_mq_w<8, 0, 2, 1, false, true>(a, n_groups, occupancy, st, tm);
  // waves per work-group: variant 17 = 4, default 8 (four waves: the Llama-shaped layer 63.8 -> 65.0 us,
  // the Qwen-shaped one 26.5 -> 27.8 us, the 86 GB context unchanged; 12 waves at 168 registers: 2 % slower)
  if (a.s.variant == 17) return launch_mq_w<4, 0, 2>(a, n_groups, occupancy, st, tm);
  // V loads carry the non-temporal hint, K loads do not (variant 20: neither).  A V row is read
  // whole by one load instruction and never again in the launch; a K row is read in 64-byte pieces
  // by four instructions, and with the hint its cache lines were sometimes dropped between them
  // (measured traffic +2.5 %).  Llama-shaped layers: 72 -> 64 us (420 MB), 460 -> 418 us (2.7 GB
  // per layer); neutral on a pool that fits the on-package cache.  Hint on K only or on both: worse.
  if (a.s.variant == 20) return launch_mq_w<8, 0, 0>(a, n_groups, occupancy, st, tm);
  if (a.s.lazy) return launch_mq_w<8, 0, 2, 1, true>(a, n_groups, occupancy, st, tm);   // the host sets lazy for the default variant only
  return launch_mq_w<8, 0, 2>(a, n_groups, occupancy, st, tm);
}

}  // namespace

int mq_row_blocks(int G, int q_len) { return G * q_len > 16 ? 2 : 1; }
int mq_heads_per_pass(int G, int q_len) {
  const int rows = 16 * mq_row_blocks(G, q_len);
  return G < rows / q_len ? G : rows / q_len;
}

hipError_t launch_attn_mq(const Shape& s, const LayerView& lv, const Scratch& sc, int q_len, const void* q,
                          const void* k_new, const void* v_new, const SeqMask& mask, const InlineLens& lens,
                          int keys_per_group, int n_groups, hipStream_t st, const KernelTimer* tm) {
  MqArgs a;
  a.s = s; a.lv = lv; a.sc = sc; a.lens = lens;
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
  a.Q = 1;
  return launch_mq_v(a, 0, out, nullptr, nullptr);
}

hipError_t launch_finish_mq(const Shape& s, const LayerView& lv, const Scratch& sc, int q_len, void* out,
                            const SeqMask& mask, const InlineLens& lens, int max_nd_eff, int keys_per_group,
                            bool narrow, hipStream_t st, const KernelTimer* tm) {
  FinishMqArgs a;
  a.s = s; a.lv = lv; a.sc = sc; a.out = out; a.mask = mask; a.lens = lens; a.inv_H = 1.0f / (float)s.H;
  a.R = keys_per_group; a.Q = q_len;
  a.HP = mq_heads_per_pass(s.G, q_len);
  a.passes = (s.G + a.HP - 1) / a.HP;
  a.RPS = 16 * mq_row_blocks(s.G, q_len);
  a.narrow = narrow ? 1 : 0;
  const int rows = s.H * q_len;
  const bool one = q_len == 1 && s.H <= 32;
  const int slots = one ? kFinishThreads : kSlotsMulti;
  dim3 grid((rows + kRowsPerBlock - 1) / kRowsPerBlock + (max_nd_eff + slots - 1) / slots, s.B);
  const size_t smem = (size_t)(rows + 2 * kFinishThreads) * sizeof(float);   // slot blocks: normalisers + exchange
  auto kern = one ? (s.lazy ? finish_mq_kernel<true, true> : finish_mq_kernel<true, false>)
                  : (s.lazy ? finish_mq_kernel<false, true> : finish_mq_kernel<false, false>);
  if (tm) hipExtLaunchKernelGGL(kern, grid, dim3(kFinishThreads), smem, st, tm->start, tm->stop, 0, a);
  else hipLaunchKernelGGL(kern, grid, dim3(kFinishThreads), smem, st, a);
  return hipGetLastError();
}

}  // namespace mkv
