// Capacity enforcement: selection of the lowest-score decode tokens (Eq. 8), removal and stable
// in-place compaction of K, V, scores and positions (Eq. 9), fired by the capacity check (Eq. 7).
// Also the token-major -> head-major ingest copy used by the prefill pool.
#include "mkv_internal.h"
#include "mkv_device.h"

#include <hip/hip_ext.h>

namespace mkv {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

using dev::ordered_key;

__device__ __forceinline__ int wave_incl_scan(int x, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int y = __shfl_up(x, off);
    if (lane >= off) x += y;
  }
  return x;
}

// Exclusive prefix sum of one int per thread over the whole block; *total gets the block sum.
__device__ __forceinline__ int block_excl_scan(int x, int* wave_sums, int* total) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int incl = wave_incl_scan(x, lane);
  __syncthreads();  // wave_sums may still be read from a previous scan
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int v = wave_sums[w];
    if (w < wave) base += v;
    tot += v;
  }
  *total = tot;
  return base + incl - x;
}

struct EvictArgs {
  Shape s;
  LayerView lv;
  Scratch sc;
  SeqMask mask;
  int threshold;
};

// One work-group per score vector (one per sequence, or one per KV head).  The pool's scores and positions sit in LDS; a 4-pass, 8-bit
// most-significant-first radix select finds the value of the overflow-th smallest candidate score;
// candidates below it leave, and of those equal to it the oldest (lowest slot = smallest position,
// because compaction is stable) leave until the count is met.  A prefix sum over the keep flags
// gives every survivor its new slot; scores and positions are rewritten from LDS, and the
// new-slot -> old-slot map is left for the row mover.
__global__ __launch_bounds__(kSelThreads) void evict_select_kernel(const EvictArgs a) {
  const Shape& s = a.s;
  const int vec = blockIdx.x;          // score vector: (sequence, vector of the sequence)
  const int b = vec / s.S;
  if (!a.mask.active(b)) return;
  const int tid = threadIdx.x;
  const int n = a.lv.nd[b];
  int* info = a.sc.evict_info + 2 * vec;
  if (n <= a.threshold || n <= s.budget) {  // Eq. 7: overflow = 0, nothing to do
    if (tid == 0) { info[0] = n; info[1] = n; }
    return;
  }
  const int k_evict = n - s.budget;   // Eq. 7
  const int n_cand = n - s.window;    // the newest `window` slots are not candidates

  extern __shared__ uint32_t smem[];
  uint32_t* raw = smem;               // [cap] score bits
  int32_t* posl = (int32_t*)(smem + s.cap);  // [cap]
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_krem, sh_first;
  __shared__ int wave_sums[kSelWaves];

  float* score = a.lv.score + (size_t)vec * s.cap;
  int32_t* pos = a.lv.pos + (size_t)vec * s.cap;
  for (int j = tid; j < n; j += kSelThreads) {
    raw[j] = __builtin_bit_cast(uint32_t, score[j]);
    posl[j] = pos[j];
  }
  if (tid == 0) { sh_prefix = 0u; sh_krem = k_evict; sh_first = n; }
  __syncthreads();

  if (k_evict == 1) {
    // The paper's own cadence (one token leaves per step once the pool is full): the selection is
    // an arg-min over (score, slot), one block-wide reduction instead of the radix passes.
    __shared__ unsigned long long wave_best[kSelWaves];
    unsigned long long best = ~0ull;
    for (int j = tid; j < n_cand; j += kSelThreads) {
      const unsigned long long v = ((unsigned long long)ordered_key(raw[j]) << 32) | (uint32_t)j;
      best = v < best ? v : best;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const unsigned long long o = __shfl_xor(best, off);
      best = o < best ? o : best;
    }
    if ((tid & 63) == 0) wave_best[tid >> 6] = best;
    __syncthreads();
    best = wave_best[0];
#pragma unroll
    for (int w = 1; w < kSelWaves; ++w) best = wave_best[w] < best ? wave_best[w] : best;
    const int e = (int)(uint32_t)best;          // the evicted slot; survivors above it move down by one
    int32_t* map1 = a.sc.src_map + (size_t)vec * s.cap;
    for (int j = e + 1 + tid; j < n; j += kSelThreads) {
      map1[j - 1] = j;
      score[j - 1] = __builtin_bit_cast(float, raw[j]);
      pos[j - 1] = posl[j];
    }
    if (tid == 0) {
      info[0] = e;
      info[1] = n - 1;   // the row mover publishes the new pool size (other vectors still read nd)
    }
    return;
  }

  // radix select: after the pass for byte `p`, sh_prefix holds the top bytes of the threshold
  // and sh_krem how many candidates to take among those that match the prefix
  for (int p = 3; p >= 0; --p) {
    const int shift = p * 8;
    const uint32_t himask = (p == 3) ? 0u : (0xffffffffu << (shift + 8));
    if (tid < 256) hist[tid] = 0u;
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    const int krem = sh_krem;
    for (int j = tid; j < n_cand; j += kSelThreads) {
      const uint32_t key = ordered_key(raw[j]);
      if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid < 64) {  // wave 0: 4 bins per lane, find the bin that holds the krem-th element
      const int c0 = hist[4 * tid], c1 = hist[4 * tid + 1], c2 = hist[4 * tid + 2], c3 = hist[4 * tid + 3];
      const int sum = c0 + c1 + c2 + c3;
      const int excl = wave_incl_scan(sum, tid) - sum;
      if (excl < krem && krem <= excl + sum) {
        int bin = 4 * tid, below = excl;
        if (below + c0 < krem) { below += c0; ++bin;
          if (below + c1 < krem) { below += c1; ++bin;
            if (below + c2 < krem) { below += c2; ++bin; } } }
        sh_prefix = prefix | ((uint32_t)bin << shift);
        sh_krem = krem - below;
      }
    }
    __syncthreads();
  }
  const uint32_t thr = sh_prefix;   // ordered key of the overflow-th smallest candidate
  const int take_eq = sh_krem;      // how many candidates equal to it leave (oldest first)

  // contiguous slots per thread so that prefix sums follow slot order
  const int items = (n + kSelThreads - 1) / kSelThreads;
  const int jb = tid * items;
  const int je = min(n, jb + items);
  int eq_cnt = 0;
  for (int j = jb; j < je; ++j) eq_cnt += (j < n_cand && ordered_key(raw[j]) == thr);
  int total;
  int eq_rank = block_excl_scan(eq_cnt, wave_sums, &total);
  int keep_cnt = 0;
  uint64_t evict_bits = 0;  // items <= 16 by the capacity limit
  for (int j = jb; j < je; ++j) {
    bool ev = false;
    if (j < n_cand) {
      const uint32_t key = ordered_key(raw[j]);
      if (key < thr) ev = true;
      else if (key == thr) { ev = eq_rank < take_eq; ++eq_rank; }
    }
    if (ev) evict_bits |= 1ull << (j - jb);
    else ++keep_cnt;
  }
  int dst = block_excl_scan(keep_cnt, wave_sums, &total);
  int first = n;
  int32_t* map = a.sc.src_map + (size_t)vec * s.cap;
  for (int j = jb; j < je; ++j) {
    if ((evict_bits >> (j - jb)) & 1ull) { first = min(first, j); continue; }
    map[dst] = j;
    score[dst] = __builtin_bit_cast(float, raw[j]);
    pos[dst] = posl[j];
    ++dst;
  }
  if (first < n) atomicMin(&sh_first, first);
  __syncthreads();
  if (tid == 0) {
    info[0] = sh_first;   // slots below the first hole stay where they are
    info[1] = total;      // = budget; published as the pool size by the row mover
  }
}

// Deferred compaction (Shape::lazy): the tokens that left are known already -- the bits of the
// vector's slot bitmap plus the selection of the last step, which has not reached the bitmap yet
// -- so this is the second half of the selection kernel alone: keep flags, prefix sum, scores and
// positions rewritten from LDS, the new-slot -> old-slot map for the row mover.  Clears the bitmap,
// the hole count and both halves of the pending selection.  One work-group per score vector.
__global__ __launch_bounds__(kSelThreads) void compact_holes_kernel(const EvictArgs a) {
  const Shape& s = a.s;
  const int vec = blockIdx.x;
  const int b = vec / s.S;
  if (!a.mask.active(b)) return;
  const int tid = threadIdx.x;
  const int n = a.lv.nd[b];
  int* info = a.sc.evict_info + 2 * vec;
  uint32_t* dead = a.lv.dead + (size_t)vec * s.capw;
  const size_t half = (size_t)s.B * s.S;
  const unsigned long long p = a.lv.pend[(size_t)(n & 1) * half + vec];
  const int pslot = p == ~0ull ? -1 : (int)(uint32_t)p;
  if (a.lv.nholes[vec] == 0 && pslot < 0) {   // nothing to close (the same for every thread)
    if (tid == 0) { info[0] = n; info[1] = n; }
    return;
  }
  extern __shared__ uint32_t smem[];
  uint32_t* raw = smem;                       // [cap] score bits
  int32_t* posl = (int32_t*)(smem + s.cap);   // [cap]
  __shared__ int sh_first;
  __shared__ int wave_sums[kSelWaves];
  float* score = a.lv.score + (size_t)vec * s.cap;
  int32_t* pos = a.lv.pos + (size_t)vec * s.cap;
  for (int j = tid; j < n; j += kSelThreads) {
    raw[j] = __builtin_bit_cast(uint32_t, score[j]);
    posl[j] = pos[j];
  }
  if (tid == 0) sh_first = n;
  const int items = (n + kSelThreads - 1) / kSelThreads;   // contiguous slots per thread: sums follow slot order
  const int jb = tid * items;
  const int je = min(n, jb + items);
  int keep_cnt = 0;
  uint64_t evict_bits = 0;                    // items <= 16 by the capacity limit
  for (int j = jb; j < je; ++j) {
    const bool ev = ((dead[j >> 5] >> (j & 31)) & 1u) || j == pslot;
    if (ev) evict_bits |= 1ull << (j - jb);
    else ++keep_cnt;
  }
  int total;
  int dst = block_excl_scan(keep_cnt, wave_sums, &total);   // (its barriers also publish raw, posl, sh_first)
  int first = n;
  int32_t* map = a.sc.src_map + (size_t)vec * s.cap;
  for (int j = jb; j < je; ++j) {
    if ((evict_bits >> (j - jb)) & 1ull) { first = min(first, j); continue; }
    map[dst] = j;
    score[dst] = __builtin_bit_cast(float, raw[j]);
    pos[dst] = posl[j];
    ++dst;
  }
  if (first < n) atomicMin(&sh_first, first);
  __syncthreads();                            // every thread has read its bitmap words
  for (int w = tid; w < s.capw; w += kSelThreads) dead[w] = 0u;
  if (tid == 0) {
    a.lv.nholes[vec] = 0;
    a.lv.pend[vec] = ~0ull;
    a.lv.pend[half + vec] = ~0ull;
    info[0] = sh_first;   // slots below the first hole stay where they are
    info[1] = total;      // live tokens; published as the pool size by the row mover
  }
}

constexpr int kMoveThreads = 1024;
constexpr int kSliceBytes = 128;
// 16 bytes in flight between a round's reads and its writes.  A native vector, not HIP's uint4
// class: arrays of the class stayed in scratch memory (144 bytes per lane by the compiler's
// resource remark), i.e. every moved row took a detour through memory.
typedef __attribute__((ext_vector_type(4))) unsigned int row16_t;

// Stable in-place row compaction.  grid (row slices, Hkv * 2, B): a work-group owns a 128-byte
// column strip of one head's K or V pool and walks the destination slots upwards.  Because a
// survivor only ever moves to a lower slot, reading a round's sources before a barrier and writing
// after it can never overwrite a row that is still to be read.
// U rows per thread and round: 8 lets a pool of up to 1024 rows move in a single round (latency
// matters there: 18 -> 8 us at 512 rows); large pools run better with one-row rounds, which
// interleave the reads and the writes of different work-groups (55 -> 45 us at 16 x 2048 rows).
template <int kMoveUnroll>
__global__ __launch_bounds__(kMoveThreads) void evict_move_kernel(const EvictArgs a, int rowb) {
  const Shape& s = a.s;
  const int b = blockIdx.z;
  if (!a.mask.active(b)) return;
  const int g = blockIdx.y >> 1;
  const int vec = b * s.S + (s.S > 1 ? g : 0);   // the score vector that governs this KV head
  const int* info = a.sc.evict_info + 2 * vec;
  const int first = info[0], n_new = info[1];
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) a.lv.nd[b] = n_new;
  if (first >= n_new) return;
  char* pool = (char*)((blockIdx.y & 1) ? a.lv.Vd : a.lv.Kd) +
               ((size_t)b * s.Hkv + g) * (size_t)s.dstride * rowb + blockIdx.x * kSliceBytes;
  const int32_t* map = a.sc.src_map + (size_t)vec * s.cap;
  constexpr int kLanesPerRow = kSliceBytes / 16;
  constexpr int kRows = kMoveThreads / kLanesPerRow;
  const int off = (threadIdx.x % kLanesPerRow) * 16;
  const int r = threadIdx.x / kLanesPerRow;
  for (int d0 = first; d0 < n_new; d0 += kRows * kMoveUnroll) {
    row16_t v[kMoveUnroll];
#pragma unroll
    for (int u = 0; u < kMoveUnroll; ++u) {
      const int d = d0 + u * kRows + r;
      v[u] = d < n_new ? *reinterpret_cast<const row16_t*>(pool + (size_t)map[d] * rowb + off) : row16_t{0u, 0u, 0u, 0u};
    }
    __builtin_amdgcn_s_waitcnt(0);  // every source of this round has arrived
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kMoveUnroll; ++u) {
      const int d = d0 + u * kRows + r;
      if (d < n_new) *reinterpret_cast<row16_t*>(pool + (size_t)d * rowb + off) = v[u];
    }
  }
}

// One-token eviction with the selection already made (the paper's cadence: one token leaves per
// step once the pool is full).  evict_key[b] holds (score key, slot) of the token that leaves, or ~0;
// every such sequence holds n = budget + 1 tokens.  Rows, scores and positions above the slot move
// down by one.  grid (row strips, Hkv * 2 + S, B): y < Hkv * 2 owns a 128-byte column strip of one
// head's K or V pool, the last S values of y (x = 0 only) a score and position vector each.  Sources of a round
// are read before a barrier and written after it, as in the general mover.
__global__ __launch_bounds__(kMoveThreads) void evict_one_kernel(const EvictArgs a, int rowb) {
  const Shape& s = a.s;
  const int b = blockIdx.z;
  if (!a.mask.active(b)) return;
  const bool rows_part = (int)blockIdx.y < s.Hkv * 2;
  const int g = blockIdx.y >> 1;
  // score vector: the one that governs this KV head, or the one whose scores this block shifts
  const int vec = b * s.S + (rows_part ? (s.S > 1 ? g : 0) : (int)blockIdx.y - s.Hkv * 2);
  const unsigned long long key = a.sc.evict_key[vec];
  if (key == ~0ull) return;
  const int e = (int)(uint32_t)key;     // the slot that leaves
  const int n_new = s.budget;
  if (!rows_part) {
    if (blockIdx.x != 0) return;
    float* score = a.lv.score + (size_t)vec * s.cap;
    int32_t* pos = a.lv.pos + (size_t)vec * s.cap;
    constexpr int kItems = kMaxDecodeCapacity / kMoveThreads;
    float sv[kItems];
    int32_t pv[kItems];
#pragma unroll
    for (int u = 0; u < kItems; ++u) {
      const int d = e + u * kMoveThreads + (int)threadIdx.x;
      sv[u] = d < n_new ? score[d + 1] : 0.f;
      pv[u] = d < n_new ? pos[d + 1] : 0;
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kItems; ++u) {
      const int d = e + u * kMoveThreads + (int)threadIdx.x;
      if (d < n_new) { score[d] = sv[u]; pos[d] = pv[u]; }
    }
    if (threadIdx.x == 0) {
      a.lv.nd[b] = n_new;
      a.sc.evict_info[2 * vec] = e;
      a.sc.evict_info[2 * vec + 1] = n_new;
    }
    return;
  }
  char* pool = (char*)((blockIdx.y & 1) ? a.lv.Vd : a.lv.Kd) +
               ((size_t)b * s.Hkv + g) * (size_t)s.dstride * rowb + blockIdx.x * kSliceBytes;
  constexpr int kLanesPerRow = kSliceBytes / 16;
  constexpr int kRows = kMoveThreads / kLanesPerRow;
  constexpr int U = 8;
  const int off = (threadIdx.x % kLanesPerRow) * 16;
  const int r = threadIdx.x / kLanesPerRow;
  for (int d0 = e; d0 < n_new; d0 += kRows * U) {
    row16_t v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int d = d0 + u * kRows + r;
      v[u] = d < n_new ? *reinterpret_cast<const row16_t*>(pool + (size_t)(d + 1) * rowb + off) : row16_t{0u, 0u, 0u, 0u};
    }
    __builtin_amdgcn_s_waitcnt(0);  // every source of this round has arrived
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int d = d0 + u * kRows + r;
      if (d < n_new) *reinterpret_cast<row16_t*>(pool + (size_t)d * rowb + off) = v[u];
    }
  }
}

// k, v [n_tokens, Hkv, D] (token-major) -> pool rows [row0, row0 + n_tokens) of every KV head of
// sequence `seq` (head-major).  One 16-byte vector per thread.
__global__ void ingest_kernel(char* Kpool, char* Vpool, const char* k, const char* v, int Hkv,
                              int rowb, int rows_cap, int seq, int row0, int n_tokens) {
  const int nv = rowb / 16;
  const size_t total = (size_t)n_tokens * Hkv * nv;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (size_t)gridDim.x * blockDim.x) {
    const int vec = (int)(i % nv);
    const size_t th = i / nv;
    const int g = (int)(th % Hkv);
    const size_t t = th / Hkv;
    const size_t dst = (((size_t)seq * Hkv + g) * rows_cap + row0 + t) * rowb + vec * 16;
    *reinterpret_cast<uint4*>(Kpool + dst) = *reinterpret_cast<const uint4*>(k + i * 16);
    *reinterpret_cast<uint4*>(Vpool + dst) = *reinterpret_cast<const uint4*>(v + i * 16);
  }
}

}  // namespace

hipError_t configure_kernels() {
  // the selection keeps scores + positions of one pool in LDS: up to 128 KiB of the CU's 160 KiB
  hipError_t e = hipFuncSetAttribute((const void*)evict_select_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDecodeCapacity * 8);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute((const void*)compact_holes_kernel,
                             hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDecodeCapacity * 8);
}

hipError_t launch_evict(const Shape& s, const LayerView& lv, const Scratch& sc, const SeqMask& mask,
                        int threshold, hipStream_t st, const KernelTimer* tm) {
  EvictArgs a;
  a.s = s; a.lv = lv; a.sc = sc; a.mask = mask; a.threshold = threshold;
  const size_t smem = (size_t)s.cap * 8;
  // with a timer: start is taken at the selection kernel, stop after the row mover
  if (tm) hipExtLaunchKernelGGL(evict_select_kernel, dim3(s.B * s.S), dim3(kSelThreads), smem, st, tm->start, nullptr, 0, a);
  else hipLaunchKernelGGL(evict_select_kernel, dim3(s.B * s.S), dim3(kSelThreads), smem, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int rowb = s.D * (s.bf16 ? 2 : 4);
  constexpr int kRowsPerPass = kMoveThreads / (kSliceBytes / 16);
  auto kern = s.budget <= kRowsPerPass * 8 ? evict_move_kernel<8> : evict_move_kernel<1>;
  const dim3 grid(rowb / kSliceBytes, s.Hkv * 2, s.B);
  if (tm) hipExtLaunchKernelGGL(kern, grid, dim3(kMoveThreads), 0, st, nullptr, tm->stop, 0, a, rowb);
  else hipLaunchKernelGGL(kern, grid, dim3(kMoveThreads), 0, st, a, rowb);
  return hipGetLastError();
}

hipError_t launch_compact_holes(const Shape& s, const LayerView& lv, const Scratch& sc, const SeqMask& mask,
                                hipStream_t st, const KernelTimer* tm) {
  EvictArgs a;
  a.s = s; a.lv = lv; a.sc = sc; a.mask = mask; a.threshold = s.budget;
  const size_t smem = (size_t)s.cap * 8;
  if (tm) hipExtLaunchKernelGGL(compact_holes_kernel, dim3(s.B * s.S), dim3(kSelThreads), smem, st, tm->start, nullptr, 0, a);
  else hipLaunchKernelGGL(compact_holes_kernel, dim3(s.B * s.S), dim3(kSelThreads), smem, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int rowb = s.D * (s.bf16 ? 2 : 4);
  constexpr int kRowsPerPass = kMoveThreads / (kSliceBytes / 16);
  auto kern = s.budget <= kRowsPerPass * 8 ? evict_move_kernel<8> : evict_move_kernel<1>;
  const dim3 grid(rowb / kSliceBytes, s.Hkv * 2, s.B);
  if (tm) hipExtLaunchKernelGGL(kern, grid, dim3(kMoveThreads), 0, st, nullptr, tm->stop, 0, a, rowb);
  else hipLaunchKernelGGL(kern, grid, dim3(kMoveThreads), 0, st, a, rowb);
  return hipGetLastError();
}

hipError_t launch_evict_one(const Shape& s, const LayerView& lv, const Scratch& sc, const SeqMask& mask,
                            hipStream_t st, const KernelTimer* tm) {
  EvictArgs a;
  a.s = s; a.lv = lv; a.sc = sc; a.mask = mask; a.threshold = s.budget;
  const int rowb = s.D * (s.bf16 ? 2 : 4);
  const dim3 grid(rowb / kSliceBytes, s.Hkv * 2 + s.S, s.B);
  if (tm) hipExtLaunchKernelGGL(evict_one_kernel, grid, dim3(kMoveThreads), 0, st, tm->start, tm->stop, 0, a, rowb);
  else hipLaunchKernelGGL(evict_one_kernel, grid, dim3(kMoveThreads), 0, st, a, rowb);
  return hipGetLastError();
}

hipError_t launch_ingest(const Shape& s, void* Kpool, void* Vpool, int rows_cap, int seq, int row0,
                         const void* k, const void* v, int n_tokens, hipStream_t st) {
  if (n_tokens <= 0) return hipSuccess;
  const int rowb = s.D * (s.bf16 ? 2 : 4);
  const size_t total = (size_t)n_tokens * s.Hkv * (rowb / 16);
  const int threads = 256;
  const int blocks = (int)((total + threads - 1) / threads < 65536 ? (total + threads - 1) / threads : 65536);
  hipLaunchKernelGGL(ingest_kernel, dim3(blocks), dim3(threads), 0, st, (char*)Kpool, (char*)Vpool,
                     (const char*)k, (const char*)v, s.Hkv, rowb, rows_cap, seq, row0, n_tokens);
  return hipGetLastError();
}

}  // namespace mkv
