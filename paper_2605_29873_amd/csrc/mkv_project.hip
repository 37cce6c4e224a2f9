// The producer of the appended token: k_t = RoPE(x_t W_k^T), v_t = x_t W_v^T for every active
// sequence, written straight into the next free slot of the decode pool (Algorithm 1, "ComputeQKV"
// followed by the append; the decode step that follows is then called without k_new / v_new).
// bf16 only.  Weights are stored as a linear layer stores them: [out features][hidden].
//
// HBM-bound on the weights (2 * Hkv * D * hidden * 2 bytes per call; the batch rides along): the
// contraction runs on v_mfma_f32_16x16x32_bf16 with a 16-feature weight tile as the A operand
// (lane (r, j) holds 8 consecutive hidden elements of feature r: one 16-byte load) and 16 sequences
// of x as the B operand.  Two launches: partial products split over the hidden axis, then a small
// kernel that adds them up, rotates and stores.
#include "mkv_internal.h"
#include "mkv_device.h"

#include <hip/hip_ext.h>

#include <math.h>

namespace mkv {
namespace {

using namespace dev;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kProjWaves = 4;        // waves per work-group, each with its own slice of the hidden axis
constexpr int kProjThreads = kProjWaves * 64;
constexpr int kBatchChunk = 64;      // sequences per pass over a wave's weight vectors

struct ProjArgs {
  Shape s;
  LayerView lv;
  SeqMask mask;
  const char* x;          // [B][hidden]
  const char* wk;         // [Hkv*D][hidden]
  const char* wv;         // [Hkv*D][hidden]
  const int32_t* rope_pos;  // [B] absolute position of the token being appended
  float* part;            // [ksplit][B][2*Hkv*D] partial sums (K features, then V features)
  int hidden;
  int ksplit;             // work-groups along the hidden axis
  double inv_freq[64];    // theta^(-2i/D), i < D/2, from the host in double precision
};

// Nearest bfloat16 (ties to even) of a double, in one rounding: going through float first would
// round twice and land on the other neighbour about once in 2^16 values.
__device__ __forceinline__ uint16_t f64_to_bf16_rne(double x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, (float)x);
  const uint32_t lo_b = u & 0xffff0000u, hi_b = lo_b + 0x10000u;   // same sign, magnitude below / above
  const double lo = (double)__builtin_bit_cast(float, lo_b), hi = (double)__builtin_bit_cast(float, hi_b);
  const double d_lo = fabs(x - lo), d_hi = fabs(hi - x);
  const bool up = d_hi < d_lo || (d_hi == d_lo && (lo_b & 0x10000u));
  return (uint16_t)((up ? hi_b : lo_b) >> 16);
}

// sin and cos of a double angle of magnitude below ~2^20, to about 1e-16: Cody-Waite reduction by
// multiples of pi/2 (the first part of pi/2 has 33 significant bits, so k * part is exact for
// |k| < 2^20), then the usual minimax polynomials on [-pi/4, pi/4].  A few dozen double FMAs; the
// library routine with its large-argument path costs an order of magnitude more, and the double
// unit is what this kernel's epilogue waits for.
// Provenance of the constants: the three-part split of pi/2 (33 + 33 + 53 bits), 2/pi and the
// minimax coefficients S1..S6 / C1..C6 are those of the public-domain fdlibm routines
// (e_rem_pio2.c, k_sin.c, k_cos.c; Sun Microsystems, 1993), the table every libm derives from;
// the code around them is this file's own.
__device__ __forceinline__ void sincos_small(double x, double* sn, double* cs) {
  const double k = rint(x * 6.36619772367581382433e-01);          // x * 2/pi
  double r = fma(-k, 1.57079632673412561417e+00, x);               // pi/2, first 33 bits
  r = fma(-k, 6.07710050630396597660e-11, r);                      // next 33 bits
  r = fma(-k, 2.02226624879595063154e-21, r);                      // the rest
  const double z = r * r;
  const double ps = -1.66666666666666324348e-01 + z * (8.33333333332248946124e-03 + z * (-1.98412698298579493134e-04 +
                    z * (2.75573137070700676789e-06 + z * (-2.50507602534068634195e-08 + z * 1.58969099521155010221e-10))));
  const double pc = 4.16666666666666019037e-02 + z * (-1.38888888888741095749e-03 + z * (2.48015872894767294178e-05 +
                    z * (-2.75573143513906633035e-07 + z * (2.08757232129817482790e-09 + z * -1.13596475577881948265e-11))));
  const double s0 = fma(r * z, ps, r);
  const double c0 = fma(z * z, pc, fma(-0.5, z, 1.0));
  const int q = (int)k & 3;
  const double s1 = (q & 1) ? c0 : s0, c1 = (q & 1) ? s0 : c0;
  *sn = (q & 2) ? -s1 : s1;
  *cs = ((q + 1) & 2) ? -c1 : c1;
}

// Stage 1: partial products.  grid (feature tiles, ksplit): a work-group contracts one 16-feature
// tile of W_k or W_v with x over 1/ksplit of the hidden axis, its four waves a quarter of that each
// (a wave requests all of its weight vectors at once: one memory latency), adds the waves up in
// LDS and leaves [16 features] x [B] partial sums.  With ksplit = 4 the launch has four work-groups
// per tile, enough to draw on every compute unit: one compute unit alone sustains only ~25 GB/s of
// this stream, so the 64 work-groups a tile-pair decomposition gives were 3x slower.
__global__ __launch_bounds__(kProjThreads) void project_partial_kernel(const ProjArgs a) {
  const Shape& s = a.s;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int r16 = lane & 15, j4 = lane >> 4;
  const int n_k = s.Hkv * s.D;                         // K features; V features follow
  const int f0 = blockIdx.x * 16;
  const int kper = a.hidden / (a.ksplit * kProjWaves);  // hidden elements per wave
  const int kbeg = (blockIdx.y * kProjWaves + wave) * kper;
  const char* W = f0 < n_k ? a.wk + (size_t)f0 * a.hidden * 2 : a.wv + (size_t)(f0 - n_k) * a.hidden * 2;
  const char* wrow = W + ((size_t)r16 * a.hidden + kbeg + 8 * j4) * 2;

  __shared__ float red[kProjWaves][16][kBatchChunk + 1];

  for (int bc = 0; bc < s.B; bc += kBatchChunk) {
    f32x4_t acc[4];
#pragma unroll
    for (int bt = 0; bt < 4; ++bt) acc[bt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const char* xrow[4];
    bool xok[4];
#pragma unroll
    for (int bt = 0; bt < 4; ++bt) {
      const int b = bc + bt * 16 + r16;
      xok[bt] = b < s.B && a.mask.active(b);
      xrow[bt] = a.x + ((size_t)(xok[bt] ? b : 0) * a.hidden + kbeg + 8 * j4) * 2;
    }
    const int live_tiles = min(4, (s.B - bc + 15) / 16);
    constexpr int CH = 8;
    for (int k0 = 0; k0 < kper; k0 += 32 * CH) {
      uint4 wa[CH];
#pragma unroll
      for (int c = 0; c < CH; ++c)
        wa[c] = (k0 + 32 * c < kper) ? ldg16(wrow + (size_t)(k0 + 32 * c) * 2) : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int bt = 0; bt < 4; ++bt) {
        if (bt < live_tiles) {
          uint4 xb[CH];
#pragma unroll
          for (int c = 0; c < CH; ++c)
            xb[c] = (xok[bt] && k0 + 32 * c < kper) ? ldg16(xrow[bt] + (size_t)(k0 + 32 * c) * 2) : make_uint4(0, 0, 0, 0);
#pragma unroll
          for (int c = 0; c < CH; ++c)
            acc[bt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wa[c]),
                                                              __builtin_bit_cast(bf16x8_t, xb[c]), acc[bt], 0, 0, 0);
        }
      }
    }
    // acc[bt][i] = partial of feature 4j + i of the tile for sequence bc + 16 bt + r
#pragma unroll
    for (int bt = 0; bt < 4; ++bt)
#pragma unroll
      for (int i = 0; i < 4; ++i) red[wave][4 * j4 + i][bt * 16 + r16] = acc[bt][i];
    __syncthreads();
    for (int item = tid; item < 16 * kBatchChunk; item += kProjThreads) {
      const int bl = item >> 4, f = item & 15;          // 16 consecutive threads: 64 contiguous bytes
      const int b = bc + bl;
      if (b < s.B) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kProjWaves; ++w) v += red[w][f][bl];
        a.part[((size_t)blockIdx.y * s.B + b) * (2 * n_k) + f0 + f] = v;
      }
    }
    __syncthreads();
  }
}

// Stage 2: one thread per (sequence, KV head, i < D/2) for K and for V: adds the ksplit partial
// sums of features i and i + D/2, rotates the K pair, rounds and stores both values into the
// sequence's next free decode slot.
//   rotation (rotate-half convention): angle_i = pos * theta^(-2i/D),
//   (k_i, k_{i+D/2}) -> (k_i cos - k_{i+D/2} sin,  k_{i+D/2} cos + k_i sin)
// The angle, sine and cosine are taken in double precision: positions reach 1e5 and a float angle
// would be off by more than a bf16 rounding step.  Positions must stay below 2^20 / max frequency,
// i.e. below about one million tokens (the host checks nothing here: rope_positions is on the device).
__global__ __launch_bounds__(256) void project_store_kernel(const ProjArgs a) {
  const Shape& s = a.s;
  const int b = blockIdx.y;
  if (!a.mask.active(b)) return;
  const int half = s.D / 2;
  const int n_k = s.Hkv * s.D;
  const int item = blockIdx.x * 256 + threadIdx.x;     // (kv, head, i)
  if (item >= 2 * s.Hkv * half) return;
  const int kv = item / (s.Hkv * half);
  const int rem = item - kv * s.Hkv * half;
  const int g = rem / half, i = rem - g * half;
  const int f = kv * n_k + g * s.D + i;
  float v0 = 0.f, v1 = 0.f;
  for (int ks = 0; ks < a.ksplit; ++ks) {
    const float* p = a.part + ((size_t)ks * s.B + b) * (2 * n_k) + f;
    v0 += p[0];
    v1 += p[half];
  }
  uint16_t o0, o1;
  if (kv == 0) {
    const double ang = (double)a.rope_pos[b] * a.inv_freq[i];
    double sn, cs;
    sincos_small(ang, &sn, &cs);
    o0 = f64_to_bf16_rne((double)v0 * cs - (double)v1 * sn);
    o1 = f64_to_bf16_rne((double)v1 * cs + (double)v0 * sn);
  } else {
    o0 = f32_to_bf16_rne(v0);
    o1 = f32_to_bf16_rne(v1);
  }
  const int slot = a.lv.nd[b];
  uint16_t* row = (uint16_t*)((char*)(kv ? a.lv.Vd : a.lv.Kd) +
                              (((size_t)b * s.Hkv + g) * (size_t)s.dstride + (size_t)slot) * (s.D * 2));
  row[i] = o0;
  row[i + half] = o1;
}

}  // namespace

int project_ksplit(int hidden) { return hidden % 512 == 0 ? 4 : 2; }

hipError_t launch_project_append(const Shape& s, const LayerView& lv, const SeqMask& mask, const void* x,
                                 const void* wk, const void* wv, const int32_t* rope_pos, float* part,
                                 int hidden, float rope_theta, hipStream_t st, const KernelTimer* tm) {
  ProjArgs a;
  a.s = s; a.lv = lv; a.mask = mask;
  a.x = (const char*)x; a.wk = (const char*)wk; a.wv = (const char*)wv;
  a.rope_pos = rope_pos; a.part = part; a.hidden = hidden; a.ksplit = project_ksplit(hidden);
  for (int i = 0; i < s.D / 2; ++i) a.inv_freq[i] = pow((double)rope_theta, -2.0 * i / s.D);
  const dim3 g1(2 * s.Hkv * s.D / 16, a.ksplit);
  const dim3 g2((2 * s.Hkv * (s.D / 2) + 255) / 256, s.B);
  if (tm) {
    hipExtLaunchKernelGGL(project_partial_kernel, g1, dim3(kProjThreads), 0, st, tm->start, nullptr, 0, a);
    hipExtLaunchKernelGGL(project_store_kernel, g2, dim3(256), 0, st, nullptr, tm->stop, 0, a);
  } else {
    hipLaunchKernelGGL(project_partial_kernel, g1, dim3(kProjThreads), 0, st, a);
    hipLaunchKernelGGL(project_store_kernel, g2, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace mkv
