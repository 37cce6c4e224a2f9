// Host side of the C ABI declared in include/mkv.h: configuration checks, arena layout,
// host mirror of the per-sequence lengths, and the launch sequence of one decode step
// (Algorithm 1).  No arithmetic of the method happens here.
#include "../../include/mkv.h"
#include "mkv_internal.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace mkv;

// Per-step scratch of mkv_decode_step_static: one array per GPU, part of the loaded code object, so
// that the entry point never allocates.  Host code may only use the address hipGetSymbolAddress
// returns for the current device (static_scratch_base below), never the array's name.
constexpr size_t kStaticScratchBytes = (size_t)MKV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up once

// Device address of the static scratch array on the current GPU (*dev_out: which one that is).
hipError_t static_scratch_base(char** out, int* dev_out = nullptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (dev_out) *dev_out = dev;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = (char*)g_scratch_ptr[dev];
  return hipSuccess;
}

constexpr size_t kAlign = 256;
constexpr int kMaxGroups = 4096;          // attention work-groups per launch, at most
// Positions of the flattened key axis charged to every unit for the fixed cost of starting a piece
// (prologue, merge): a work-group whose range crosses a unit boundary gets that many keys fewer,
// which evens out the finishing times.  Against no charge at all: batch-1 Llama layer 11.4 -> 9.0 us
// attention, Qwen-shaped layer 26.7 -> 25.0 us, ragged Llama layer 63.9 -> 63.1 us, the 86 GB
// context unchanged.  Swept again 128 .. 512 beside the tail pad below (two runs each, one box):
// ragged Llama layer 71.7 / 71.9 / 72.2 / 72.4 / 72.9 / 73.0 us per step at 128 / 192 / 256 / 320 /
// 384 / 512, Qwen-shaped layer 34.4 / 33.9 / 34.0 / 34.0 / 34.3 / 34.5, batch-1 layer flat.
constexpr int kPiecePad = 192;
// Virtual positions behind every unit's keys, for the extra work of the work-group that takes the
// unit's end: the decode keys' logits are staged in LDS and written out, the appended rows are read
// from the caller's tensors, marked slots are masked.  Swept 0 / 64 / 96 / 128 (three runs each,
// one box): Qwen-shaped layer 35.9 / 34.9 / 34.7 / 34.1 us per step, ragged Llama layer 72.0 / 71.9 /
// 72.1 / 72.1, batch-1 layer 16.0 / 15.8 / 15.9 / 15.9; a surcharge proportional to the decode pool
// (a quarter of a position per slot and more) helped the Qwen shape as much and cost the ragged
// Llama layer 1 us and more.
constexpr int kTailPad = 128;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  // per-layer regions (byte offsets inside a layer block) and the layer stride
  size_t Kp, Vp, Kd, Vd, score, pos, mlen, nd, nd_eff, tpos, dead, nholes, pend, layer_bytes;
  // scratch regions (absolute offsets), shared by all layers
  size_t part_o, part_ml, offs, logits, abar, lse, src_map, evict_info, evict_key, total;
  size_t p_score, p_pos, p_map, p_info;   // prompt compression: one sequence at a time
  size_t proj_part;                       // partial sums of the fused k/v projection (bf16 contexts)
  int cap, HL, passes, max_groups;
  int S;                  // score vectors per sequence
  int mq_passes;          // most passes per KV head on the matrix-core kernels (0: they are not used)
  int mq_slot_rows;       // most rows per partial slot on the matrix-core kernels
  bool mfma_single;       // mkv_decode_step runs on the matrix-core kernels
  int pstride, dstride;   // padded row strides of the (seq, kv head) regions
  bool lazy;              // one-token evictions are deferred: slot bitmap + compaction every few dozen steps
  int capw;               // words of one score vector's slot bitmap
};

// Deferred compaction applies at the paper's cadence (trigger == budget: one token leaves per
// step) on the default matrix-core kernels, single-query steps only.
bool cadence_on_matrix_cores(const mkv_config* c) {
  return c->evict_trigger == c->decode_budget && c->max_q_len == 0 && c->dtype == MKV_BF16 &&
         c->head_dim == 128 && c->attn_variant == 0;
}

// decode_capacity == 0: one append past the trigger -- plus, where compaction is deferred, room
// for the evicted tokens' slots between two compactions (an eighth of the budget, 8..64 slots:
// the dead rows are still streamed by the attention kernel, so the room is kept small).
int64_t default_capacity(const mkv_config* c) {
  const int64_t grow = c->max_q_len > 1 ? c->max_q_len : 1;
  int64_t cap = (int64_t)c->evict_trigger + grow;
  if (cadence_on_matrix_cores(c)) {
    int64_t slack = c->decode_budget / 8;
    slack = slack < 8 ? 8 : slack > 64 ? 64 : slack;
    if (cap + slack <= kMaxDecodeCapacity) cap += slack;
  }
  return cap;
}

thread_local std::string g_create_error;

std::string fmt(const char* f, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, f);
  vsnprintf(buf, sizeof buf, f, ap);
  va_end(ap);
  return buf;
}

// Returns an empty string when cfg is usable, else the reason.
std::string check_config(const mkv_config* c) {
  if (!c) return "cfg is NULL";
  if (c->n_layers < 1 || c->batch < 1) return "n_layers and batch must be >= 1";
  if (c->batch > kMaxBatch) return fmt("batch %d above the supported %d", c->batch, kMaxBatch);
  if (c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads != 0)
    return "n_q_heads must be a positive multiple of n_kv_heads";
  if (c->head_dim != 64 && c->head_dim != 128) return "head_dim must be 64 or 128";
  if (c->dtype != MKV_F32 && c->dtype != MKV_BF16) return "dtype must be MKV_F32 or MKV_BF16";
  if (c->max_prefill < 0) return "max_prefill must be >= 0";
  // one (sequence, KV head) region is addressed with 32-bit byte offsets
  if ((int64_t)c->max_prefill * c->head_dim * 4 >= (int64_t)1 << 31)
    return "max_prefill * head_dim must stay below 2^29 elements per KV head";
  if (c->decode_budget < 1) return "decode_budget must be >= 1";
  if (c->evict_trigger < c->decode_budget) return "evict_trigger must be >= decode_budget";
  if (c->recent_window < 0 || c->recent_window > c->decode_budget)
    return "recent_window must lie in [0, decode_budget]";
  if (!(c->alpha >= 0.0f && c->alpha <= 1.0f)) return "alpha must lie in [0, 1]";
  if (!(c->softmax_scale >= 0.0f) || isinf(c->softmax_scale)) return "softmax_scale must be finite and >= 0";
  if (c->score_mode != MKV_SCORE_LAYER_MEAN && c->score_mode != MKV_SCORE_PER_KV_HEAD) return "unknown score_mode";
  if (c->split_keys < 0 || (c->split_keys % 16) != 0 || (c->split_keys && c->split_keys < 64))
    return "split_keys must be 0 or a multiple of 16 that is at least 64";
  if (c->attn_variant < 0 || c->attn_variant > 32) return "attn_variant out of range";
  if (c->groups_per_cu < 0 || c->groups_per_cu > 16) return "groups_per_cu out of range";
  if (c->max_q_len < 0 || c->max_q_len > 16) return "max_q_len must lie in [0, 16]";
  if (c->max_q_len > 0 && (c->dtype != MKV_BF16 || c->head_dim != 128))
    return "max_q_len > 0 needs MKV_BF16 and head_dim 128";
  const int64_t grow = c->max_q_len > 1 ? c->max_q_len : 1;   // most tokens one call appends
  int64_t cap = c->decode_capacity;
  if (cap == 0) {
    if (c->evict_trigger == MKV_NEVER_EVICT) return "decode_capacity is required with MKV_NEVER_EVICT";
    cap = default_capacity(c);
  }
  if (cap <= c->decode_budget) return "decode_capacity must exceed decode_budget";
  if (c->evict_trigger != MKV_NEVER_EVICT && cap < (int64_t)c->evict_trigger + grow)
    return "decode_capacity must be at least evict_trigger + max(1, max_q_len)";
  if (cap > kMaxDecodeCapacity) return fmt("decode capacity %lld above the supported %d", (long long)cap, kMaxDecodeCapacity);
  if (c->arena && ((uintptr_t)c->arena % kAlign) != 0) return "arena must be 256-byte aligned";
  return "";
}

Layout make_layout(const mkv_config* c) {
  Layout L;
  memset(&L, 0, sizeof L);
  const int grow = c->max_q_len > 1 ? c->max_q_len : 1;
  const int G = c->n_q_heads / c->n_kv_heads;
  L.S = c->score_mode == MKV_SCORE_PER_KV_HEAD ? c->n_kv_heads : 1;
  L.cap = c->decode_capacity ? c->decode_capacity : (int)default_capacity(c);
  L.lazy = cadence_on_matrix_cores(c) && L.cap > c->decode_budget + 1;
  L.capw = L.cap / 32 + 2;      // two spare words: a tile's 32 bits are cut out of two consecutive words
  L.HL = head_lanes(G);
  L.passes = (G + L.HL - 1) / L.HL;
  // Single-query steps of bf16 x 128 layers run on the matrix-core kernels as well: the vector-ALU
  // kernel spends G multiply-adds per loaded element and falls behind the memory stream as G grows
  // (measured at G = 7: 3.7 -> 5.1 TB/s; at G = 4: 5.4 -> 5.6 TB/s).  attn_variant 1..15 forces the
  // vector-ALU kernel, 16.. picks a variant of the matrix-core one.
  const bool mfma_ok = c->dtype == MKV_BF16 && c->head_dim == 128;
  L.mfma_single = mfma_ok && (c->attn_variant == 0 || c->attn_variant >= 16);
  if (c->max_q_len > 0 || L.mfma_single) {
    // most passes per KV head and most rows per partial slot over the call lengths in use
    for (int ql = 1; ql <= grow; ++ql) {
      if (ql > 1 && c->max_q_len == 0) break;
      const int hp = mq_heads_per_pass(G, ql);
      const int ps = (G + hp - 1) / hp;
      if (ps > L.mq_passes) L.mq_passes = ps;
      if (16 * mq_row_blocks(G, ql) > L.mq_slot_rows) L.mq_slot_rows = 16 * mq_row_blocks(G, ql);
    }
  }
  const size_t es = c->dtype == MKV_BF16 ? 2 : 4;
  const size_t B = c->batch, Hkv = c->n_kv_heads, H = c->n_q_heads, D = c->head_dim;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  // each (seq, kv head) region is followed by 4 KiB of padding: with power-of-two region sizes the
  // work-groups that run side by side would otherwise all hit the same memory channels (measured:
  // +10 % attention bandwidth on the ragged 16-sequence Llama layer)
  const int pad_rows = (int)(4096 / (D * es));
  L.pstride = c->max_prefill ? c->max_prefill + pad_rows : 0;
  L.dstride = L.cap + pad_rows;
  L.Kp = take(B * Hkv * (size_t)L.pstride * D * es);
  L.Vp = take(B * Hkv * (size_t)L.pstride * D * es);
  L.Kd = take(B * Hkv * (size_t)L.dstride * D * es);
  L.Vd = take(B * Hkv * (size_t)L.dstride * D * es);
  L.score = take(B * L.S * L.cap * 4);
  L.pos = take(B * L.S * L.cap * 4);
  L.mlen = take(B * 4);
  L.nd = take(B * 4);
  L.nd_eff = take(B * 4);
  L.tpos = take(B * 4);
  L.dead = take(B * L.S * (size_t)L.capw * 4);
  L.nholes = take(B * L.S * 4);
  L.pend = take(2 * B * L.S * 8);       // starts at all ones (no selection pending), the rest at zero
  L.layer_bytes = o;
  o = L.layer_bytes * (size_t)c->n_layers;
  // a work-group takes at least 64 keys, so small pools never need many partial slots
  const size_t most_passes = L.passes > L.mq_passes ? L.passes : L.mq_passes;
  const size_t key_cap = B * Hkv * most_passes * ((size_t)c->max_prefill + L.cap);
  L.max_groups = (int)(key_cap / 64 + 1 < (size_t)kMaxGroups ? key_cap / 64 + 1 : (size_t)kMaxGroups);
  const size_t slots = (size_t)L.max_groups + B * Hkv * L.passes;
  const size_t mq_slots = L.mq_passes ? (size_t)L.max_groups + B * Hkv * L.mq_passes : 0;
  const size_t rows = slots * L.HL > mq_slots * L.mq_slot_rows ? slots * L.HL : mq_slots * L.mq_slot_rows;   // partial rows
  L.part_o = take(rows * D * 4);
  L.part_ml = take(rows * 2 * 4);
  L.offs = take((B + 1) * 8);
  L.logits = take(B * H * grow * (((size_t)L.cap + 63) / 64 * 64) * 4);   // the matrix-core path tiles the slot axis by 64
  L.abar = take(B * L.S * L.cap * 4);
  L.lse = take(B * H * grow * 4);
  L.src_map = take(B * L.S * L.cap * 4);
  L.evict_info = take(B * L.S * 2 * 4);
  L.evict_key = take(B * L.S * 8);
  if (c->max_prefill > 0 && c->max_prefill <= kMaxDecodeCapacity) {
    L.p_score = take((size_t)c->max_prefill * 4);
    L.p_pos = take((size_t)c->max_prefill * 4);
    L.p_map = take((size_t)c->max_prefill * 4);
    L.p_info = take(4 * 4);      // (first moved slot, new size), then the row count the kernels read
  }
  if (c->dtype == MKV_BF16) L.proj_part = take((size_t)4 * B * 2 * Hkv * D * 4);
  L.total = o;
  return L;
}

__global__ void set_int_kernel(int32_t* p, int32_t v) { *p = v; }
__global__ void iota_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i;
}

}  // namespace

// Event-bracketed kernel timing, off unless mkv_set_profiling asked for it.
struct Profiler {
  static constexpr int kSlots = 512;       // steps recorded before the sums are folded
  bool on = false;
  std::vector<hipEvent_t> ev;              // 6 events per slot: start/stop of attention, finish, eviction
  std::vector<uint8_t> evicted;
  int used = 0;
  double us[3] = {0, 0, 0};
  int64_t steps = 0, evict_steps = 0;
};

struct mkv_ctx {
  mkv_config cfg;
  Layout lay;
  Shape shape;
  hipStream_t stream;
  int device;            // the GPU that was current in mkv_create: arena, stream and kernels live there
  char* arena;
  bool own_arena;
  // [L*B]; h_nd: decode slots in use, of which h_holes hold evicted tokens that await compaction
  // (deferred compaction only); h_last_n, h_last_slots [B]: live tokens and slots the last step saw
  std::vector<int32_t> h_mlen, h_nd, h_holes, h_last_n, h_last_slots;
  std::vector<uint8_t> probs_compacted;  // [B]: compacted since the last step: its per-slot head means are gone
  bool poisoned;         // a launch failed in the middle of a step: device state and mirror may differ
  std::vector<int64_t> h_step;
  std::vector<uint8_t> frozen;
  std::vector<uint8_t> in_pool;   // [L*B]: mkv_project_append has written the next token's row already
  int last_layer;
  int view;            // score vector the read/write helpers address (mkv_set_score_view)
  int last_q_len;      // query rows of the step taken last
  Scratch last_sc;     // scratch the last decode step ran on (mkv_read_probs reads it back)
  int target_groups;   // attention work-groups a launch aims for: compute units x groups per unit
  int mq_target_groups;  // same for the multi-query kernel
  std::string err;
  Profiler prof;
};

namespace {

int fail(mkv_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->err = msg; else g_create_error = msg;
  return code;
}
int fail_hip(mkv_ctx* ctx, hipError_t e, const char* what) {
  return fail(ctx, MKV_ERR_HIP, fmt("%s: %s", what, hipGetErrorString(e)));
}
// A HIP error after part of a call's work has been enqueued: the device's bookkeeping and the host
// mirror may no longer agree, so the context refuses every further call but mkv_destroy.
int poison(mkv_ctx* ctx, hipError_t e, const char* what) {
  ctx->poisoned = true;
  return fail_hip(ctx, e, what);
}
// First line of every entry point that uses the cache state.
int refuse_if_poisoned(mkv_ctx* ctx) {
  return ctx->poisoned ? fail(ctx, MKV_ERR_STATE, "an earlier call failed half-way (MKV_ERR_HIP): the context can only be destroyed")
                       : MKV_OK;
}

LayerView layer_view(const mkv_ctx* c, int layer) {
  char* base = c->arena + c->lay.layer_bytes * (size_t)layer;
  LayerView v;
  v.Kp = base + c->lay.Kp; v.Vp = base + c->lay.Vp;
  v.Kd = base + c->lay.Kd; v.Vd = base + c->lay.Vd;
  v.score = (float*)(base + c->lay.score);
  v.pos = (int32_t*)(base + c->lay.pos);
  v.mlen = (int32_t*)(base + c->lay.mlen);
  v.nd = (int32_t*)(base + c->lay.nd);
  v.nd_eff = (int32_t*)(base + c->lay.nd_eff);
  v.tpos = (int32_t*)(base + c->lay.tpos);
  v.dead = (uint32_t*)(base + c->lay.dead);
  v.nholes = (int32_t*)(base + c->lay.nholes);
  v.pend = (unsigned long long*)(base + c->lay.pend);
  return v;
}

Scratch scratch_view(const mkv_ctx* c) {
  Scratch s;
  s.part_o = (float*)(c->arena + c->lay.part_o);
  s.part_ml = (float*)(c->arena + c->lay.part_ml);
  s.offs = (long long*)(c->arena + c->lay.offs);
  s.logits = (float*)(c->arena + c->lay.logits);
  s.abar = (float*)(c->arena + c->lay.abar);
  s.lse = (float*)(c->arena + c->lay.lse);
  s.src_map = (int32_t*)(c->arena + c->lay.src_map);
  s.evict_info = (int32_t*)(c->arena + c->lay.evict_info);
  s.evict_key = (unsigned long long*)(c->arena + c->lay.evict_key);
  return s;
}

// The scratch of one decode step laid out in the static array instead of the arena: the same
// regions as in make_layout, sized for this launch (`slots` partial slots of `rows` rows, `q_len`
// query rows per sequence).  Returns the bytes needed; fills *out when they fit.
size_t carve_static(const mkv_ctx* c, char* base, size_t slots, int rows, int q_len, Scratch* out) {
  const size_t B = c->cfg.batch, H = c->cfg.n_q_heads, D = c->cfg.head_dim, S = c->lay.S, cap = c->lay.cap;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  const size_t part_o = take(slots * rows * D * 4);
  const size_t part_ml = take(slots * rows * 2 * 4);
  const size_t offs = take((B + 1) * 8);
  const size_t logits = take(B * H * q_len * ((cap + 63) / 64 * 64) * 4);
  const size_t abar = take(B * S * cap * 4);
  const size_t lse = take(B * H * q_len * 4);
  const size_t src_map = take(B * S * cap * 4);
  const size_t evict_info = take(B * S * 2 * 4);
  const size_t evict_key = take(B * S * 8);
  if (o <= kStaticScratchBytes) {
    out->part_o = (float*)(base + part_o);
    out->part_ml = (float*)(base + part_ml);
    out->offs = (long long*)(base + offs);
    out->logits = (float*)(base + logits);
    out->abar = (float*)(base + abar);
    out->lse = (float*)(base + lse);
    out->src_map = (int32_t*)(base + src_map);
    out->evict_info = (int32_t*)(base + evict_info);
    out->evict_key = (unsigned long long*)(base + evict_key);
  }
  return o;
}

constexpr int kEvPerSlot = 6;

// Folds the recorded slots into the sums (waits for the stream to drain first).
hipError_t prof_fold(mkv_ctx* c) {
  Profiler& p = c->prof;
  if (p.used == 0) return hipSuccess;
  hipError_t e = hipStreamSynchronize(c->stream);
  for (int i = 0; i < p.used && e == hipSuccess; ++i) {
    hipEvent_t* q = &p.ev[(size_t)i * kEvPerSlot];
    float ms[3] = {0, 0, 0};
    e = hipEventElapsedTime(&ms[0], q[0], q[1]);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms[1], q[2], q[3]);
    if (e == hipSuccess && p.evicted[i]) e = hipEventElapsedTime(&ms[2], q[4], q[5]);
    for (int k = 0; k < 3; ++k) p.us[k] += 1000.0 * ms[k];
    p.steps += 1;
    p.evict_steps += p.evicted[i];
  }
  p.used = 0;
  return e;
}

// Device tensors are read and written in 16-byte vectors.
bool misaligned(const void* p) { return ((uintptr_t)p & 15) != 0; }

bool bad_index(const mkv_ctx* c, int layer, int seq) {
  return layer < 0 || layer >= c->cfg.n_layers || seq < 0 || seq >= c->cfg.batch;
}

int set_device_int(mkv_ctx* c, int32_t* p, int32_t v) {
  hipLaunchKernelGGL(set_int_kernel, dim3(1), dim3(1), 0, c->stream, p, v);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MKV_OK : fail_hip(c, e, "set_int launch");
}

// Deferred compaction: closes the holes of the masked sequences that have any (one launch pair for
// the layer).  Afterwards their slots in use equal their live tokens.
int flush_holes(mkv_ctx* c, int layer, const SeqMask& mask, const Scratch& sc, const KernelTimer* tm = nullptr,
                bool* fired = nullptr) {
  if (fired) *fired = false;
  if (!c->lay.lazy) return MKV_OK;
  const int B = c->cfg.batch;
  SeqMask todo;
  memset(&todo, 0, sizeof todo);
  bool any = false;
  for (int b = 0; b < B; ++b)
    if (mask.active(b) && c->h_holes[(size_t)layer * B + b] > 0) {
      todo.w[b >> 6] |= 1ull << (b & 63);
      any = true;
    }
  if (!any) return MKV_OK;
  hipError_t e = launch_compact_holes(c->shape, layer_view(c, layer), sc, todo, c->stream, tm);
  if (e != hipSuccess) return poison(c, e, "compaction launch");
  for (int b = 0; b < B; ++b)
    if (todo.active(b)) {
      const size_t i = (size_t)layer * B + b;
      c->h_nd[i] -= c->h_holes[i];
      c->h_holes[i] = 0;
      if (layer == c->last_layer) c->probs_compacted[b] = 1;
    }
  if (fired) *fired = true;
  return MKV_OK;
}

SeqMask one_seq(int b) {
  SeqMask m;
  memset(&m, 0, sizeof m);
  m.w[b >> 6] |= 1ull << (b & 63);
  return m;
}

// Evicts the sequences of `mask` whose mirror length exceeds `threshold`; returns MKV_OK when no
// sequence qualifies.
// `selected`: the finishing kernel of the step just taken may have left the one-token selection
// (single-query step with trigger == budget); it is used when every sequence that fires holds
// exactly budget + 1 tokens.
int run_evict(mkv_ctx* c, int layer, const SeqMask& mask, int threshold, const Scratch& sc, bool* fired = nullptr,
              const KernelTimer* tm = nullptr, bool selected = false) {
  const int B = c->cfg.batch;
  bool any = false;
  for (int b = 0; b < B; ++b) {
    const int n = c->h_nd[(size_t)layer * B + b];
    if (mask.active(b) && n > threshold && n > c->cfg.decode_budget) {
      any = true;
      if (n != c->cfg.decode_budget + 1) selected = false;
    }
  }
  if (fired) *fired = any;
  if (!any) return MKV_OK;
  hipError_t e = selected ? launch_evict_one(c->shape, layer_view(c, layer), sc, mask, c->stream, tm)
                          : launch_evict(c->shape, layer_view(c, layer), sc, mask, threshold, c->stream, tm);
  if (e != hipSuccess) return poison(c, e, "evict launch");
  for (int b = 0; b < B; ++b) {
    int32_t& n = c->h_nd[(size_t)layer * B + b];
    if (mask.active(b) && n > threshold && n > c->cfg.decode_budget) n = c->cfg.decode_budget;
  }
  return MKV_OK;
}

// One pass of Algorithm 1 over the active sequences of a layer, appending q_len tokens per
// sequence; `mq` selects the multi-query kernels (q, k_new, v_new and out then carry q_len rows per
// sequence).
// `static_scratch`: the step's scratch is the per-GPU static array instead of the arena's regions.
int step(mkv_ctx* c, int layer, int q_len, bool mq, const void* q, const void* k_new, const void* v_new,
         void* out, const uint8_t* seq_mask, bool static_scratch = false) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, MKV_ERR_ARG, "layer out of range");
  if (!q || !out) return fail(c, MKV_ERR_ARG, "q and out must not be NULL");
  if ((k_new == nullptr) != (v_new == nullptr)) return fail(c, MKV_ERR_ARG, "k_new and v_new must be given together");
  if (misaligned(q) || misaligned(out) || misaligned(k_new) || misaligned(v_new))
    return fail(c, MKV_ERR_ARG, "q, k_new, v_new and out must be 16-byte aligned");
  const bool rows_in_pool = k_new == nullptr;   // mkv_project_append has produced the new rows
  if (rows_in_pool && q_len != 1) return fail(c, MKV_ERR_ARG, "k_new and v_new must not be NULL");
  const int B = c->cfg.batch;
  const int G = c->cfg.n_q_heads / c->cfg.n_kv_heads;
  int passes = c->lay.passes;
  if (mq) {
    const int hp = mq_heads_per_pass(G, q_len);
    passes = (G + hp - 1) / hp;
  }
  const int P = unit_extra(c->shape);   // virtual positions per unit: the fixed costs of a piece and of a unit's end
  const bool lazy = c->lay.lazy;
  // 1. checks; nothing is changed before all of them have passed
  SeqMask mask;
  memset(&mask, 0, sizeof mask);
  int n_active = 0;
  bool need_room = false;              // deferred compaction: some sequence's slots are used up by holes
  for (int b = 0; b < B; ++b) {
    if (seq_mask && !seq_mask[b]) continue;
    const size_t i = (size_t)layer * B + b;
    if ((c->in_pool[i] != 0) != rows_in_pool)
      return fail(c, MKV_ERR_STATE, rows_in_pool
                  ? fmt("sequence %d: no row from mkv_project_append is waiting, k_new and v_new are needed", b)
                  : fmt("sequence %d: mkv_project_append has appended this step's row, pass k_new = v_new = NULL", b));
    if (c->h_nd[i] + q_len > c->lay.cap) {
      if (c->h_nd[i] - c->h_holes[i] + q_len > c->lay.cap)
        return fail(c, MKV_ERR_CAPACITY, fmt("sequence %d: %d of %d decode slots used, %d more needed", b,
                                             c->h_nd[i] - c->h_holes[i], c->lay.cap, q_len));
      need_room = true;
    }
    mask.w[b >> 6] |= 1ull << (b & 63);
    ++n_active;
  }
  if (n_active == 0) return MKV_OK;
  hipEvent_t* pe = nullptr;
  KernelTimer t_attn, t_fin, t_ev;
  if (c->prof.on) {
    if (c->prof.used == Profiler::kSlots) {
      hipError_t pe_err = prof_fold(c);
      if (pe_err != hipSuccess) return fail_hip(c, pe_err, "profile events");
    }
    pe = &c->prof.ev[(size_t)c->prof.used * kEvPerSlot];
    c->prof.evicted[c->prof.used] = 0;
    t_attn = {pe[0], pe[1]}; t_fin = {pe[2], pe[3]}; t_ev = {pe[4], pe[5]};
  }
  // work-groups of the attention launch for a flattened key axis of `total` positions
  const int target = mq ? c->mq_target_groups : c->target_groups;
  auto plan = [&](long long total, long long* R_out) -> long long {
    long long R = c->cfg.split_keys ? c->cfg.split_keys : (total + target - 1) / target;
    if (R < 64) R = 64;       // a work-group takes at least 64 positions (sizes the partial buffers)
    const long long r_min = (total + c->lay.max_groups - 1) / c->lay.max_groups;
    if (R < r_min) R = r_min;
    *R_out = R;
    return (total + R - 1) / R;
  };
  char* static_base = nullptr;
  if (static_scratch) {
    int dev_now = -1;
    hipError_t se = static_scratch_base(&static_base, &dev_now);
    if (se != hipSuccess) return fail_hip(c, se, "address of the static scratch array");
    // every GPU has its own copy of the array: the one of another GPU is no memory of this context's
    if (dev_now != c->device)
      return fail(c, MKV_ERR_STATE, fmt("GPU %d is current, the context was created on GPU %d", dev_now, c->device));
    // does the step's scratch fit?  Decided here, before anything is enqueued, on the slots in use
    // now: a compaction below can only shorten the key axis
    long long total_now = 0, R_now = 0;
    for (int b = 0; b < B; ++b)
      if (mask.active(b)) {
        const size_t i = (size_t)layer * B + b;
        total_now += (long long)c->cfg.n_kv_heads * passes * (c->h_mlen[i] + c->h_nd[i] + q_len + P);
      }
    // (a shorter axis may split into a few more ranges, never more than the launch's target)
    long long groups_most = plan(total_now, &R_now);
    if (groups_most < target) groups_most = target;
    const size_t slots = (size_t)groups_most + (size_t)B * c->cfg.n_kv_heads * passes;
    Scratch probe;
    const size_t need = carve_static(c, static_base, slots, mq ? 16 * mq_row_blocks(G, q_len) : c->lay.HL, q_len, &probe);
    if (need > kStaticScratchBytes)
      return fail(c, MKV_ERR_CAPACITY, fmt("this step needs %zu bytes of scratch, the static array holds %zu: use "
                                           "mkv_decode_step", need, kStaticScratchBytes));
  }
  // 2. deferred compaction: a sequence whose slots are used up gets its holes closed first (the
  //    live tokens stay what they are; only their slots change)
  bool timed_evict = false;
  if (need_room) {
    Scratch fsc = scratch_view(c);
    if (static_scratch) (void)carve_static(c, static_base, 0, 1, q_len, &fsc);   // fits: it is part of the step's
    bool fired = false;
    int frc = flush_holes(c, layer, mask, fsc, pe ? &t_ev : nullptr, &fired);
    if (frc != MKV_OK) return frc;
    timed_evict = fired;
  }
  // 3. lengths, flattened key axis
  InlineLens lens;
  memset(&lens, 0, sizeof lens);
  lens.valid = B <= kInlineLens;
  int max_n1 = 0;
  long long total_keys = 0;  // length of the flattened key axis of this launch
  for (int b = 0; b < B; ++b) {
    const size_t i = (size_t)layer * B + b;
    if (lens.valid) {
      lens.mlen[b] = c->h_mlen[i];
      lens.nd[b] = c->h_nd[i];
    }
    if (!mask.active(b)) continue;
    const int n1 = c->h_nd[i] + q_len;
    total_keys += (long long)c->cfg.n_kv_heads * passes * (c->h_mlen[i] + n1 + P);
    if (n1 > max_n1) max_n1 = n1;
  }
  if (lens.valid) {
    long long run = 0;
    for (int b = 0; b < B; ++b) {
      lens.offs[b] = run;
      if (mask.active(b)) run += (long long)c->cfg.n_kv_heads * passes * (lens.mlen[b] + lens.nd[b] + q_len + P);
    }
    lens.offs[B] = run;
  }
  LayerView lv = layer_view(c, layer);
  // equal key ranges, one per work-group: as many work-groups as the chip holds at once, unless
  // the caller fixed the range length.  The length is not rounded: with sequences of equal length
  // and a unit count that divides (or is divided by) the work-group count, every range then starts
  // and ends on unit boundaries and no work-group pays for two pieces (the 86 GB context, 256
  // units on 256 work-groups: 419 -> 406 us per layer); a range may start and end at any key.
  long long R = 0;
  const int n_groups = (int)plan(total_keys, &R);
  if (R > INT32_MAX - 63) return fail(c, MKV_ERR_CAPACITY, "key range per work-group overflows");
  hipError_t e;
  Scratch sc = scratch_view(c);
  if (static_scratch) {
    // partial slots this launch can touch: one per work-group plus one per (sequence, KV head, pass)
    const size_t slots = (size_t)n_groups + (size_t)B * c->cfg.n_kv_heads * passes;
    const int rows = mq ? 16 * mq_row_blocks(G, q_len) : c->lay.HL;
    if (carve_static(c, static_base, slots, rows, q_len, &sc) > kStaticScratchBytes)    // checked above
      return fail(c, MKV_ERR_CAPACITY, "static scratch");
  }
  if (mq) e = launch_attn_mq(c->shape, lv, sc, q_len, q, k_new, v_new, mask, lens, (int)R, n_groups, c->stream, pe ? &t_attn : nullptr);
  else e = launch_attn(c->shape, lv, sc, q, k_new, v_new, mask, (int)R, n_groups, c->stream, pe ? &t_attn : nullptr);
  if (e != hipSuccess) return poison(c, e, "attention launch");
  if (mq) e = launch_finish_mq(c->shape, lv, sc, q_len, out, mask, lens, max_n1, (int)R, total_keys < (1ll << 31), c->stream, pe ? &t_fin : nullptr);
  else e = launch_finish(c->shape, lv, sc, out, mask, max_n1, (int)R, c->stream, pe ? &t_fin : nullptr);
  if (e != hipSuccess) return poison(c, e, "finish launch");
  for (int b = 0; b < B; ++b) {
    if (!mask.active(b)) continue;
    const size_t i = (size_t)layer * B + b;
    c->h_nd[i] += q_len;
    c->h_step[i] += q_len;
    c->frozen[i] = 1;
    c->in_pool[i] = 0;
    c->h_last_n[b] = c->h_nd[i] - c->h_holes[i];
    c->h_last_slots[b] = c->h_nd[i];
  }
  c->last_layer = layer;
  c->last_q_len = q_len;
  c->last_sc = sc;
  std::fill(c->probs_compacted.begin(), c->probs_compacted.end(), (uint8_t)0);
  int rc = MKV_OK;
  if (c->cfg.evict_trigger != MKV_NEVER_EVICT) {
    bool fired = false;
    if (lazy) {
      // The finishing kernel has taken the one-token selection of every sequence that holds
      // budget + 1 live tokens (Eq. 7-8); the token's slot is only marked (Eq. 9 follows at the next
      // compaction).  Anything further over budget -- possible after mkv_load_decode -- goes
      // through the general selection, on a pool without holes.
      bool general = false;
      for (int b = 0; b < B; ++b) {
        if (!mask.active(b)) continue;
        const size_t i = (size_t)layer * B + b;
        const int live = c->h_nd[i] - c->h_holes[i];
        if (live == c->cfg.decode_budget + 1) c->h_holes[i] += 1;
        else if (live > c->cfg.decode_budget) general = true;
      }
      if (general) {
        rc = flush_holes(c, layer, mask, sc);
        if (rc == MKV_OK) rc = run_evict(c, layer, mask, c->cfg.evict_trigger, sc, &fired, (pe && !timed_evict) ? &t_ev : nullptr, false);
      }
    } else {
      const bool selected = q_len == 1 && c->cfg.evict_trigger == c->cfg.decode_budget;
      rc = run_evict(c, layer, mask, c->cfg.evict_trigger, sc, &fired, pe ? &t_ev : nullptr, selected);
    }
    if (fired) timed_evict = true;
  }
  if (pe && timed_evict) c->prof.evicted[c->prof.used] = 1;
  if (pe) c->prof.used += 1;
  return rc;
}

}  // namespace

extern "C" {

size_t mkv_required_bytes(const mkv_config* cfg) {
  if (!check_config(cfg).empty()) return 0;
  return make_layout(cfg).total;
}

int mkv_create(const mkv_config* cfg, mkv_ctx** out) {
  if (!out) return fail(nullptr, MKV_ERR_ARG, "out is NULL");
  *out = nullptr;
  std::string why = check_config(cfg);
  if (!why.empty()) return fail(nullptr, MKV_ERR_ARG, why);
  mkv_ctx* c = new (std::nothrow) mkv_ctx();
  if (!c) return fail(nullptr, MKV_ERR_NOMEM, "host allocation failed");
  c->cfg = *cfg;
  c->lay = make_layout(cfg);
  c->stream = (hipStream_t)cfg->stream;
  c->last_layer = -1;
  c->last_q_len = 1;
  c->view = 0;
  c->poisoned = false;
  if (cfg->arena) {
    if (cfg->arena_bytes < c->lay.total) {
      std::string m = fmt("arena of %zu bytes given, %zu needed", cfg->arena_bytes, c->lay.total);
      delete c;
      return fail(nullptr, MKV_ERR_NOMEM, m);
    }
    c->arena = (char*)cfg->arena;
    c->own_arena = false;
  } else {
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, c->lay.total);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      std::string m = fmt("hipMalloc of %zu bytes: %s", c->lay.total, hipGetErrorString(e));
      delete c;
      return fail(nullptr, MKV_ERR_NOMEM, m);
    }
    c->arena = (char*)p;
    c->own_arena = true;
  }
  Shape& s = c->shape;
  s.B = cfg->batch; s.H = cfg->n_q_heads; s.Hkv = cfg->n_kv_heads; s.G = s.H / s.Hkv;
  s.D = cfg->head_dim; s.bf16 = cfg->dtype == MKV_BF16;
  s.max_prefill = cfg->max_prefill; s.cap = c->lay.cap; s.pstride = c->lay.pstride; s.dstride = c->lay.dstride; s.HL = c->lay.HL; s.passes = c->lay.passes; s.max_groups = c->lay.max_groups;
  s.budget = cfg->decode_budget; s.window = cfg->recent_window; s.alpha = cfg->alpha;
  s.trigger = cfg->evict_trigger; s.S = c->lay.S;
  s.variant = cfg->attn_variant;
  s.piece_pad = kPiecePad;
  s.tail_pad = kTailPad;
  s.lazy = c->lay.lazy ? 1 : 0;
  s.capw = c->lay.capw;
  const double scale = cfg->softmax_scale > 0.f ? (double)cfg->softmax_scale : 1.0 / sqrt((double)s.D);
  s.scale_log2 = (float)(scale * 1.4426950408889634074);
  const size_t LB = (size_t)cfg->n_layers * cfg->batch;
  c->h_mlen.assign(LB, 0); c->h_nd.assign(LB, 0); c->h_holes.assign(LB, 0); c->h_step.assign(LB, 0); c->frozen.assign(LB, 0); c->in_pool.assign(LB, 0);
  c->h_last_n.assign(cfg->batch, 0);
  c->h_last_slots.assign(cfg->batch, 0);
  c->probs_compacted.assign(cfg->batch, 0);
  c->last_sc = scratch_view(c);
  hipError_t e = configure_kernels();
  c->device = -1;
  if (e == hipSuccess) {   // address of the static scratch array on this GPU, for mkv_decode_step_static
    char* base = nullptr;
    e = static_scratch_base(&base, &c->device);
  }
  {
    int dev = 0, cus = 256;
    if (e == hipSuccess) e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    // one launch = exactly the work-groups the chip holds at once (registers and LDS decide)
    int per_cu = cfg->groups_per_cu;
    if (per_cu == 0 && e == hipSuccess) e = attn_groups_per_cu(c->shape, &per_cu);
    if (per_cu < 1) per_cu = 1;
    c->target_groups = cus * per_cu;
    if (c->target_groups > c->lay.max_groups) c->target_groups = c->lay.max_groups;
    c->mq_target_groups = 0;
    if (c->lay.mq_passes > 0) {
      int mq_per_cu = cfg->groups_per_cu;
      if (mq_per_cu == 0 && e == hipSuccess) e = attn_mq_groups_per_cu(c->shape, &mq_per_cu);
      if (mq_per_cu < 1) mq_per_cu = 1;
      c->mq_target_groups = cus * mq_per_cu;
      if (c->mq_target_groups > c->lay.max_groups) c->mq_target_groups = c->lay.max_groups;
    }
  }
  // bookkeeping starts at zero: scores, positions, all lengths, the scratch
  for (int l = 0; l < cfg->n_layers && e == hipSuccess; ++l) {
    char* base = c->arena + c->lay.layer_bytes * (size_t)l;
    e = hipMemsetAsync(base + c->lay.score, 0, c->lay.pend - c->lay.score, c->stream);
    if (e == hipSuccess)     // no selection pending: all ones
      e = hipMemsetAsync(base + c->lay.pend, 0xFF, c->lay.layer_bytes - c->lay.pend, c->stream);
  }
  if (e == hipSuccess)
    e = hipMemsetAsync(c->arena + c->lay.part_o, 0, c->lay.total - c->lay.part_o, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) {
    std::string m = fmt("context initialisation: %s", hipGetErrorString(e));
    if (c->own_arena) (void)hipFree(c->arena);
    delete c;
    return fail(nullptr, MKV_ERR_HIP, m);
  }
  *out = c;
  return MKV_OK;
}

int mkv_destroy(mkv_ctx* c) {
  if (!c) return MKV_OK;
  hipError_t e = hipStreamSynchronize(c->stream);
  for (hipEvent_t ev : c->prof.ev) (void)hipEventDestroy(ev);
  if (c->own_arena) {
    hipError_t e2 = hipFree(c->arena);
    if (e == hipSuccess) e = e2;
  }
  delete c;
  return e == hipSuccess ? MKV_OK : MKV_ERR_HIP;
}

int mkv_prefill_append(mkv_ctx* c, int layer, int seq, const void* k, const void* v, int n_tokens) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (bad_index(c, layer, seq)) return fail(c, MKV_ERR_ARG, "layer or seq out of range");
  if (n_tokens < 0 || (n_tokens > 0 && (!k || !v))) return fail(c, MKV_ERR_ARG, "k/v NULL or n_tokens < 0");
  if (misaligned(k) || misaligned(v)) return fail(c, MKV_ERR_ARG, "k and v must be 16-byte aligned");
  const size_t i = (size_t)layer * c->cfg.batch + seq;
  if (c->frozen[i]) return fail(c, MKV_ERR_FROZEN, "prefill pool is frozen after the first decode step");
  if ((int64_t)c->h_mlen[i] + n_tokens > c->cfg.max_prefill)
    return fail(c, MKV_ERR_CAPACITY, fmt("prefill %d + %d exceeds max_prefill %d", c->h_mlen[i], n_tokens, c->cfg.max_prefill));
  if (n_tokens == 0) return MKV_OK;
  LayerView lv = layer_view(c, layer);
  hipError_t e = launch_ingest(c->shape, lv.Kp, lv.Vp, c->lay.pstride, seq, c->h_mlen[i], k, v, n_tokens, c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "ingest launch");
  int rc = set_device_int(c, lv.mlen + seq, c->h_mlen[i] + n_tokens);
  if (rc != MKV_OK) { c->poisoned = true; return rc; }    // rows are in the pool, the length is not
  c->h_mlen[i] += n_tokens;
  return MKV_OK;
}

int mkv_prefill_compress(mkv_ctx* c, int layer, int seq, const float* token_scores, int keep) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (bad_index(c, layer, seq)) return fail(c, MKV_ERR_ARG, "layer or seq out of range");
  if (!token_scores || keep < 1) return fail(c, MKV_ERR_ARG, "token_scores NULL or keep < 1");
  const size_t i = (size_t)layer * c->cfg.batch + seq;
  if (c->frozen[i]) return fail(c, MKV_ERR_FROZEN, "prefill pool is frozen after the first decode step");
  const int M = c->h_mlen[i];
  if (keep >= M) return MKV_OK;
  if (c->cfg.max_prefill > kMaxDecodeCapacity)
    return fail(c, MKV_ERR_CAPACITY, fmt("prompt compression handles pools of up to %d tokens (max_prefill is %d)",
                                         kMaxDecodeCapacity, c->cfg.max_prefill));
  // The selection and compaction kernels of the decode pool, pointed at this sequence's prefill
  // pool: one sequence, one score vector, budget = keep, no protected window.
  Shape s = c->shape;
  s.B = 1; s.S = 1; s.cap = c->cfg.max_prefill; s.dstride = c->lay.pstride;
  s.budget = keep; s.window = 0; s.trigger = MKV_NEVER_EVICT; s.lazy = 0;
  LayerView lv = layer_view(c, layer);
  const size_t rowb = (size_t)c->cfg.head_dim * (c->cfg.dtype == MKV_BF16 ? 2 : 4);
  const size_t seq_off = (size_t)seq * c->cfg.n_kv_heads * c->lay.pstride * rowb;
  int32_t* info = (int32_t*)(c->arena + c->lay.p_info);
  LayerView pv = lv;
  pv.Kd = (char*)lv.Kp + seq_off; pv.Vd = (char*)lv.Vp + seq_off;
  pv.score = (float*)(c->arena + c->lay.p_score);
  pv.pos = (int32_t*)(c->arena + c->lay.p_pos);
  pv.nd = info + 2;
  Scratch sc = scratch_view(c);
  sc.src_map = (int32_t*)(c->arena + c->lay.p_map);
  sc.evict_info = info;
  hipError_t e = hipMemcpyAsync(pv.score, token_scores, (size_t)M * 4, hipMemcpyDeviceToDevice, c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "copy of the token scores");
  hipLaunchKernelGGL(iota_kernel, dim3((M + 255) / 256), dim3(256), 0, c->stream, pv.pos, M);
  e = hipGetLastError();
  if (e != hipSuccess) return fail_hip(c, e, "iota launch");
  int rc = set_device_int(c, pv.nd, M);
  if (rc != MKV_OK) return rc;
  SeqMask mask;
  memset(&mask, 0, sizeof mask);
  mask.w[0] = 1ull;
  e = launch_evict(s, pv, sc, mask, keep, c->stream);
  if (e != hipSuccess) return poison(c, e, "prompt compression launch");
  rc = set_device_int(c, lv.mlen + seq, keep);
  if (rc != MKV_OK) { c->poisoned = true; return rc; }
  c->h_mlen[i] = keep;
  return MKV_OK;
}

int mkv_project_append(mkv_ctx* c, int layer, const void* x, const void* w_k, const void* w_v, int hidden,
                       const int32_t* rope_positions, float rope_theta, const uint8_t* seq_mask) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, MKV_ERR_ARG, "layer out of range");
  if (!x || !w_k || !w_v || !rope_positions) return fail(c, MKV_ERR_ARG, "x, w_k, w_v and rope_positions must not be NULL");
  if (misaligned(x) || misaligned(w_k) || misaligned(w_v)) return fail(c, MKV_ERR_ARG, "x, w_k and w_v must be 16-byte aligned");
  if (c->cfg.dtype != MKV_BF16) return fail(c, MKV_ERR_ARG, "mkv_project_append needs MKV_BF16");
  if (hidden < 256 || hidden % 256 != 0) return fail(c, MKV_ERR_ARG, "hidden must be a positive multiple of 256");
  if (!(rope_theta > 1.0f) || isinf(rope_theta)) return fail(c, MKV_ERR_ARG, "rope_theta must be finite and above 1");
  const int B = c->cfg.batch;
  SeqMask mask;
  memset(&mask, 0, sizeof mask);
  int n_active = 0;
  bool need_room = false;
  for (int b = 0; b < B; ++b) {
    if (seq_mask && !seq_mask[b]) continue;
    const size_t i = (size_t)layer * B + b;
    if (c->in_pool[i]) return fail(c, MKV_ERR_STATE, fmt("sequence %d: the previous projected row has not been consumed by a decode step", b));
    if (c->h_nd[i] - c->h_holes[i] >= c->lay.cap)
      return fail(c, MKV_ERR_CAPACITY, fmt("sequence %d: decode pool is full (%d slots)", b, c->lay.cap));
    if (c->h_nd[i] >= c->lay.cap) need_room = true;
    mask.w[b >> 6] |= 1ull << (b & 63);
    ++n_active;
  }
  if (n_active == 0) return MKV_OK;
  if (need_room) {       // deferred compaction: the row needs a free slot at the end of the pool
    int frc = flush_holes(c, layer, mask, scratch_view(c));
    if (frc != MKV_OK) return frc;
  }
  hipError_t e = launch_project_append(c->shape, layer_view(c, layer), mask, x, w_k, w_v, rope_positions,
                                       (float*)(c->arena + c->lay.proj_part), hidden, rope_theta, c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "projection launch");
  for (int b = 0; b < B; ++b)
    if (mask.active(b)) c->in_pool[(size_t)layer * B + b] = 1;
  return MKV_OK;
}

int mkv_decode_step(mkv_ctx* c, int layer, const void* q, const void* k_new, const void* v_new,
                    void* out, const uint8_t* seq_mask) {
  return step(c, layer, 1, c && c->lay.mfma_single, q, k_new, v_new, out, seq_mask);
}

int mkv_decode_step_static(mkv_ctx* c, int layer, const void* q, const void* k_new, const void* v_new,
                           void* out, const uint8_t* seq_mask) {
  return step(c, layer, 1, c && c->lay.mfma_single, q, k_new, v_new, out, seq_mask, true);
}

int mkv_decode_step_multi(mkv_ctx* c, int layer, int q_len, const void* q, const void* k_new,
                          const void* v_new, void* out, const uint8_t* seq_mask) {
  if (!c) return MKV_ERR_ARG;
  if (c->cfg.max_q_len == 0) return fail(c, MKV_ERR_STATE, "the context was created with max_q_len = 0");
  if (q_len < 1 || q_len > c->cfg.max_q_len)
    return fail(c, MKV_ERR_ARG, fmt("q_len %d outside [1, max_q_len = %d]", q_len, c->cfg.max_q_len));
  return step(c, layer, q_len, true, q, k_new, v_new, out, seq_mask);
}

int mkv_evict(mkv_ctx* c, int layer, int seq) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (layer < 0 || layer >= c->cfg.n_layers || seq < -1 || seq >= c->cfg.batch)
    return fail(c, MKV_ERR_ARG, "layer or seq out of range");
  SeqMask mask;
  memset(&mask, 0, sizeof mask);
  for (int b = 0; b < c->cfg.batch; ++b) {
    if (seq >= 0 && b != seq) continue;
    if (c->in_pool[(size_t)layer * c->cfg.batch + b])
      return fail(c, MKV_ERR_STATE, fmt("sequence %d: a projected row is waiting for its decode step", b));
    mask.w[b >> 6] |= 1ull << (b & 63);
  }
  int rc = flush_holes(c, layer, mask, scratch_view(c));
  if (rc != MKV_OK) return rc;
  return run_evict(c, layer, mask, c->cfg.decode_budget, scratch_view(c));
}

int mkv_read_scores(mkv_ctx* c, int layer, int seq, float* scores, int32_t* positions, int capacity,
                    int* n_out) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (bad_index(c, layer, seq)) return fail(c, MKV_ERR_ARG, "layer or seq out of range");
  const size_t i = (size_t)layer * c->cfg.batch + seq;
  {   // readers see the pool in order of generation without holes
    int frc = flush_holes(c, layer, one_seq(seq), scratch_view(c));
    if (frc != MKV_OK) return frc;
  }
  LayerView lv = layer_view(c, layer);
  int32_t n_dev = -1;
  hipError_t e = hipMemcpyAsync(&n_dev, lv.nd + seq, 4, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "read pool size");
  if (n_dev != c->h_nd[i])
    return fail(c, MKV_ERR_STATE, fmt("device pool size %d differs from the host mirror %d", n_dev, c->h_nd[i]));
  if (n_out) *n_out = n_dev;
  if ((scores || positions) && capacity < n_dev) return fail(c, MKV_ERR_CAPACITY, "buffer too small");
  if (scores && n_dev) e = hipMemcpyAsync(scores, lv.score + ((size_t)seq * c->lay.S + c->view) * c->lay.cap, (size_t)n_dev * 4, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess && positions && n_dev)
    e = hipMemcpyAsync(positions, lv.pos + ((size_t)seq * c->lay.S + c->view) * c->lay.cap, (size_t)n_dev * 4, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "read scores");
  return MKV_OK;
}

int mkv_write_scores(mkv_ctx* c, int layer, int seq, const float* scores, int n) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (bad_index(c, layer, seq) || !scores) return fail(c, MKV_ERR_ARG, "bad index or NULL scores");
  const size_t i = (size_t)layer * c->cfg.batch + seq;
  if (n != c->h_nd[i] - c->h_holes[i]) return fail(c, MKV_ERR_ARG, fmt("n = %d but the pool holds %d", n, c->h_nd[i] - c->h_holes[i]));
  if (n == 0) return MKV_OK;
  {
    int frc = flush_holes(c, layer, one_seq(seq), scratch_view(c));
    if (frc != MKV_OK) return frc;
  }
  LayerView lv = layer_view(c, layer);
  hipError_t e = hipMemcpyAsync(lv.score + ((size_t)seq * c->lay.S + c->view) * c->lay.cap, scores, (size_t)n * 4, hipMemcpyHostToDevice, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "write scores");
  return MKV_OK;
}

int mkv_load_decode(mkv_ctx* c, int layer, int seq, const void* k, const void* v, const float* scores,
                    const int32_t* positions, int n, int64_t next_step) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (bad_index(c, layer, seq)) return fail(c, MKV_ERR_ARG, "layer or seq out of range");
  if (n < 0 || (n > 0 && (!k || !v || !scores || !positions))) return fail(c, MKV_ERR_ARG, "NULL input or n < 0");
  if (misaligned(k) || misaligned(v)) return fail(c, MKV_ERR_ARG, "k and v must be 16-byte aligned");
  if (n > c->lay.cap) return fail(c, MKV_ERR_CAPACITY, fmt("n = %d above the decode capacity %d", n, c->lay.cap));
  if (next_step < 0 || next_step > INT32_MAX) return fail(c, MKV_ERR_ARG, "next_step out of range");
  for (int j = 0; j < n; ++j) {
    if (positions[j] < 0 || positions[j] >= next_step || (j && positions[j] <= positions[j - 1]))
      return fail(c, MKV_ERR_ARG, "positions must be strictly increasing and below next_step");
  }
  const size_t i = (size_t)layer * c->cfg.batch + seq;
  LayerView lv = layer_view(c, layer);
  hipError_t e = launch_ingest(c->shape, lv.Kd, lv.Vd, c->lay.dstride, seq, 0, k, v, n, c->stream);
  for (int sv = 0; sv < c->lay.S && n; ++sv) {   // every score vector starts from the same snapshot
    const size_t vec = (size_t)seq * c->lay.S + sv;
    if (e == hipSuccess) e = hipMemcpyAsync(lv.score + vec * c->lay.cap, scores, (size_t)n * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(lv.pos + vec * c->lay.cap, positions, (size_t)n * 4, hipMemcpyHostToDevice, c->stream);
  }
  if (e == hipSuccess && c->lay.lazy) {     // no holes, no selection pending
    const size_t v0 = (size_t)seq * c->lay.S, half = (size_t)c->cfg.batch * c->lay.S;
    e = hipMemsetAsync(lv.dead + v0 * c->lay.capw, 0, (size_t)c->lay.S * c->lay.capw * 4, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(lv.nholes + v0, 0, (size_t)c->lay.S * 4, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(lv.pend + v0, 0xFF, (size_t)c->lay.S * 8, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(lv.pend + half + v0, 0xFF, (size_t)c->lay.S * 8, c->stream);
  }
  if (e != hipSuccess) return poison(c, e, "load decode pool");
  int rc = set_device_int(c, lv.nd + seq, n);
  if (rc == MKV_OK) rc = set_device_int(c, lv.tpos + seq, (int32_t)next_step);
  if (rc != MKV_OK) { c->poisoned = true; return rc; }
  e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return poison(c, e, "load decode pool");
  c->h_nd[i] = n;
  c->h_holes[i] = 0;
  c->h_step[i] = next_step;
  c->frozen[i] = 1;
  c->in_pool[i] = 0;
  return MKV_OK;
}

int mkv_read_kv(mkv_ctx* c, int layer, int seq, int pool, int kv_head, void* k, void* v, int capacity,
                int* n_out) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (bad_index(c, layer, seq) || kv_head < 0 || kv_head >= c->cfg.n_kv_heads || (pool != 0 && pool != 1))
    return fail(c, MKV_ERR_ARG, "bad layer, seq, pool or kv_head");
  const size_t i = (size_t)layer * c->cfg.batch + seq;
  if (pool == 0) {
    int frc = flush_holes(c, layer, one_seq(seq), scratch_view(c));
    if (frc != MKV_OK) return frc;
  }
  const int n = pool ? c->h_mlen[i] : c->h_nd[i];
  if (n_out) *n_out = n;
  if ((k || v) && capacity < n) return fail(c, MKV_ERR_CAPACITY, "buffer too small");
  LayerView lv = layer_view(c, layer);
  const size_t rowb = (size_t)c->cfg.head_dim * (c->cfg.dtype == MKV_BF16 ? 2 : 4);
  const size_t rows = pool ? (size_t)c->lay.pstride : (size_t)c->lay.dstride;
  const size_t off = ((size_t)seq * c->cfg.n_kv_heads + kv_head) * rows * rowb;
  hipError_t e = hipSuccess;
  if (k && n) e = hipMemcpyAsync(k, (char*)(pool ? lv.Kp : lv.Kd) + off, n * rowb, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess && v && n)
    e = hipMemcpyAsync(v, (char*)(pool ? lv.Vp : lv.Vd) + off, n * rowb, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "read kv");
  return MKV_OK;
}

int mkv_read_probs(mkv_ctx* c, int layer, int seq, float* abar, float* lse_per_head, int capacity,
                   int* n_out) {
  if (!c) return MKV_ERR_ARG;
  if (bad_index(c, layer, seq)) return fail(c, MKV_ERR_ARG, "layer or seq out of range");
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (layer != c->last_layer) return fail(c, MKV_ERR_STATE, "layer was not the layer stepped last");
  const int n = c->h_last_n[seq];
  if (n_out) *n_out = n;
  if (abar && capacity < n) return fail(c, MKV_ERR_CAPACITY, "buffer too small");
  const Scratch& sc = c->last_sc;
  hipError_t e = hipSuccess;
  const size_t vec = (size_t)seq * c->lay.S + c->view;
  const int slots = c->h_last_slots[seq];
  if (abar && n && slots != n) {
    // deferred compaction: the step wrote one value per slot; the slots of tokens that had left
    // before the step are dropped here (the step's own selection was still part of its pool)
    if (c->probs_compacted[seq])
      return fail(c, MKV_ERR_STATE, "the pool has been compacted since the step: its head means are gone");
    std::vector<float> per_slot((size_t)slots);
    std::vector<uint32_t> dead((size_t)c->lay.capw);
    e = hipMemcpyAsync(per_slot.data(), sc.abar + vec * c->lay.cap, (size_t)slots * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess)
      e = hipMemcpyAsync(dead.data(), layer_view(c, layer).dead + vec * c->lay.capw, (size_t)c->lay.capw * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return fail_hip(c, e, "read probs");
    int k = 0;
    for (int j = 0; j < slots; ++j)
      if (!((dead[j >> 5] >> (j & 31)) & 1u) && k < n) abar[k++] = per_slot[j];
    if (k != n) return fail(c, MKV_ERR_STATE, fmt("%d live slots found, %d expected", k, n));
  } else if (abar && n) {
    e = hipMemcpyAsync(abar, sc.abar + vec * c->lay.cap, (size_t)n * 4, hipMemcpyDeviceToHost, c->stream);
  }
  if (e == hipSuccess && lse_per_head) {
    // [B][q_len][H]: the last query row of the sequence
    const size_t row = (size_t)seq * c->last_q_len + (c->last_q_len - 1);
    e = hipMemcpyAsync(lse_per_head, sc.lse + row * c->cfg.n_q_heads, (size_t)c->cfg.n_q_heads * 4, hipMemcpyDeviceToHost, c->stream);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "read probs");
  if (lse_per_head)
    for (int h = 0; h < c->cfg.n_q_heads; ++h) lse_per_head[h] *= 0.69314718055994530942f;  // base 2 -> e
  return MKV_OK;
}

int mkv_read_slots(mkv_ctx* c, int layer, int seq, float* scores, int32_t* positions, uint8_t* live,
                   int capacity, int* n_slots, int* pending_slot) {
  if (!c) return MKV_ERR_ARG;
  if (refuse_if_poisoned(c)) return MKV_ERR_STATE;
  if (bad_index(c, layer, seq)) return fail(c, MKV_ERR_ARG, "layer or seq out of range");
  const size_t i = (size_t)layer * c->cfg.batch + seq;
  const int n = c->h_nd[i];
  if (n_slots) *n_slots = n;
  if (pending_slot) *pending_slot = -1;
  if ((scores || positions || live) && capacity < n) return fail(c, MKV_ERR_CAPACITY, "buffer too small");
  LayerView lv = layer_view(c, layer);
  const size_t vec = (size_t)seq * c->lay.S + c->view;
  hipError_t e = hipSuccess;
  std::vector<uint32_t> dead;
  unsigned long long pend = ~0ull;
  if (scores && n) e = hipMemcpyAsync(scores, lv.score + vec * c->lay.cap, (size_t)n * 4, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess && positions && n)
    e = hipMemcpyAsync(positions, lv.pos + vec * c->lay.cap, (size_t)n * 4, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess && c->lay.lazy) {
    dead.resize((size_t)c->lay.capw);
    e = hipMemcpyAsync(dead.data(), lv.dead + vec * c->lay.capw, (size_t)c->lay.capw * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess)    // the half that belongs to a pool of n slots
      e = hipMemcpyAsync(&pend, lv.pend + (size_t)(n & 1) * c->cfg.batch * c->lay.S + vec, 8, hipMemcpyDeviceToHost, c->stream);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "read slots");
  if (live)
    for (int j = 0; j < n; ++j) live[j] = dead.empty() ? 1 : !((dead[j >> 5] >> (j & 31)) & 1u);
  if (pending_slot && pend != ~0ull) *pending_slot = (int)(uint32_t)pend;
  return MKV_OK;
}

int mkv_set_score_view(mkv_ctx* c, int kv_head) {
  if (!c) return MKV_ERR_ARG;
  if (kv_head < 0 || kv_head >= c->lay.S) return fail(c, MKV_ERR_ARG, fmt("score vector %d outside [0, %d)", kv_head, c->lay.S));
  c->view = kv_head;
  return MKV_OK;
}

int mkv_get_lens(mkv_ctx* c, int layer, int seq, int* n_prefill, int* n_decode, int64_t* step) {
  if (!c) return MKV_ERR_ARG;
  if (bad_index(c, layer, seq)) return fail(c, MKV_ERR_ARG, "layer or seq out of range");
  const size_t i = (size_t)layer * c->cfg.batch + seq;
  if (n_prefill) *n_prefill = c->h_mlen[i];
  if (n_decode) *n_decode = c->h_nd[i] - c->h_holes[i];
  if (step) *step = c->h_step[i];
  return MKV_OK;
}

int mkv_set_profiling(mkv_ctx* c, int enable) {
  if (!c) return MKV_ERR_ARG;
  Profiler& p = c->prof;
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return fail_hip(c, e, "stream synchronize");
  if (enable && p.ev.empty()) {
    p.ev.resize((size_t)Profiler::kSlots * kEvPerSlot);
    p.evicted.assign(Profiler::kSlots, 0);
    for (size_t i = 0; i < p.ev.size(); ++i) {
      e = hipEventCreate(&p.ev[i]);
      if (e != hipSuccess) {
        for (size_t k = 0; k < i; ++k) (void)hipEventDestroy(p.ev[k]);
        p.ev.clear();
        return fail_hip(c, e, "hipEventCreate");
      }
    }
  }
  p.on = enable != 0;
  p.used = 0;
  p.us[0] = p.us[1] = p.us[2] = 0.0;
  p.steps = p.evict_steps = 0;
  return MKV_OK;
}

int mkv_read_profile(mkv_ctx* c, double* kernel_us, int64_t* counts) {
  if (!c) return MKV_ERR_ARG;
  hipError_t e = prof_fold(c);
  if (e != hipSuccess) return fail_hip(c, e, "profile events");
  if (kernel_us) for (int k = 0; k < 3; ++k) kernel_us[k] = c->prof.us[k];
  if (counts) { counts[0] = c->prof.steps; counts[1] = c->prof.evict_steps; }
  return MKV_OK;
}

const char* mkv_last_error(const mkv_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
