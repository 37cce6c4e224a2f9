// Internal declarations shared by the library's own translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mkv {

constexpr int kMaxBatch = 1024;          // sequences per layer (mask is passed by value)
constexpr int kMaxDecodeCapacity = 16384;  // the selection kernel keeps one pool in LDS
constexpr int kMaskWords = kMaxBatch / 64;

// Which sequences take part in a launch; passed by value so a step needs no host->device copy.
struct SeqMask {
  uint64_t w[kMaskWords];
  __host__ __device__ bool active(int b) const { return (w[b >> 6] >> (b & 63)) & 1ull; }
};

// Per-sequence lengths from the host's mirror, by value with the launch when the batch is small:
// the kernels then start without a round trip to memory for them.
constexpr int kInlineLens = 32;
struct InlineLens {
  int32_t mlen[kInlineLens];   // prefill length M
  int32_t nd[kInlineLens];     // decode pool size before the step
  long long offs[kInlineLens + 1];  // start of each sequence on the launch's flattened key axis
  int32_t valid;               // 0: read the lengths from LayerView instead
};

// Shapes and parameters of a context, by value to every kernel.
struct Shape {
  int B, H, Hkv, G, D, bf16;
  int max_prefill;   // row capacity of the prefill pool per (seq, kv head)
  int cap;           // row capacity of the decode pool per (seq, kv head)
  int pstride;       // rows between consecutive (seq, kv head) regions of the prefill pool
  int dstride;       // same for the decode pool (>= cap; padded, see the arena layout)
  int HL;            // query heads one attention pass serves per KV head: 1, 2, 4 or 8
  int passes;        // passes per KV head: ceil(G / HL)
  int max_groups;    // most attention work-groups a launch may use (sizes the partial buffers)
  int S;             // score vectors per sequence: 1 (mean over all query heads) or Hkv (one per KV head)
  int budget, window;
  int trigger;       // the decode step evicts when the pool exceeds this (INT32_MAX: never)
  int variant;       // attention kernel variant (tuning), 0 = default
  int piece_pad;     // positions of the flattened key axis charged to a unit for starting a piece
  int tail_pad;      // virtual positions behind a unit's keys: the work-group that takes the end of a unit
                     // -- the decode keys -- also stages and writes their logits and reads the appended
                     // rows, so it gets that many keys fewer
  int lazy;          // 1: one-token evictions only mark the slot (LayerView::dead) and the rows are
                     //    compacted every few dozen steps; 0: every eviction compacts at once
  int capw;          // 32-bit words of one score vector's slot bitmap (LayerView::dead)
  float alpha;
  float scale_log2;  // softmax scale * log2(e): logits are kept in base-2 units
};

// One layer's slice of the arena.  Pools are head-major: [B][Hkv][rows][D].
struct LayerView {
  void* Kp; void* Vp;      // prefill pool
  void* Kd; void* Vd;      // decode pool
  float* score;            // [B][S][cap]   importance vector(s) I
  int32_t* pos;            // [B][S][cap]   original decode position of each slot (per vector: with
                           //               S = Hkv the KV heads retain different tokens)
  int32_t* mlen;           // [B]        prefill length M
  int32_t* nd;             // [B]        decode pool size before the step in flight
  int32_t* nd_eff;         // [B]        decode pool size including the token appended in this step
  int32_t* tpos;           // [B]        decode steps taken = position the next token gets
  // Deferred compaction (Shape::lazy).  A slot whose token has been evicted keeps its rows until
  // the next compaction; the attention kernel masks it, the finishing kernel skips it.
  uint32_t* dead;          // [B][S][capw]  bit j set: slot j holds an evicted token
  int32_t* nholes;         // [B][S]        number of bits set in the vector's bitmap
  // [2][B][S]: selection key (score key, slot) of the one-token eviction taken by the step that
  // brought the pool to n slots sits in half n & 1 (~0: none).  The next step's attention kernel
  // masks that slot and moves it into the bitmap.
  unsigned long long* pend;
};

// Per-step scratch, shared by all layers (layers run one after another on one stream).
struct Scratch {
  // per piece: un-normalised partial outputs and (reference, sum) pairs in base-2 units; HL rows
  // per slot in the single-query kernels, 16 in the multi-query ones
  float* part_o;      // [max_groups + B*Hkv*passes][HL][D]
  float* part_ml;     // [max_groups + B*Hkv*passes][HL][2]
  long long* offs;    // [B+1]  prefix sums of the per-sequence key counts of the last launch
  float* logits;      // base-2 logits of decode keys: [B][H][cap] on the vector-ALU path,
                      // [B][ceil(cap/64)][H*q_len][64] on the matrix-core path
  float* abar;        // [B][S][cap]       head-mean decode-slice attention of the last step
  float* lse;         // [B][q_len][H]     base-2 log of the softmax normaliser of the last step
  int32_t* src_map;   // [B][S][cap]       compaction map: new slot -> old slot
  int32_t* evict_info;  // [B][S][2]       (first moved slot, new pool size) of the last selection
  // [B][S] when the step will evict exactly one token per sequence (trigger == budget): the finishing
  // kernel's arg-min over (score, slot) of the candidates, ~0 if the sequence is not over budget
  unsigned long long* evict_key;
};

// Events that bracket one kernel launch (start and stop are recorded by the launch itself).
struct KernelTimer { hipEvent_t start, stop; };

hipError_t launch_ingest(const Shape& s, void* Kpool, void* Vpool, int rows_cap, int seq, int row0,
                         const void* k, const void* v, int n_tokens, hipStream_t st);

hipError_t launch_attn(const Shape& s, const LayerView& lv, const Scratch& sc, const void* q,
                       const void* k_new, const void* v_new, const SeqMask& mask, int keys_per_group,
                       int n_groups, hipStream_t st, const KernelTimer* tm = nullptr);

// How many attention work-groups of this shape's kernel variant are resident per compute unit.
hipError_t attn_groups_per_cu(const Shape& s, int* out);

hipError_t launch_finish(const Shape& s, const LayerView& lv, const Scratch& sc, void* out,
                         const SeqMask& mask, int max_nd_eff, int keys_per_group, hipStream_t st,
                         const KernelTimer* tm = nullptr);

// Evicts every masked sequence whose pool size exceeds `threshold` back to s.budget.
hipError_t launch_evict(const Shape& s, const LayerView& lv, const Scratch& sc, const SeqMask& mask,
                        int threshold, hipStream_t st, const KernelTimer* tm = nullptr);

// Multi-query step (bf16, head_dim 128): q_len query rows per sequence on the matrix cores.
// A pass serves mq_heads_per_pass(G, q_len) query heads x q_len rows per KV head, in
// mq_row_blocks(G, q_len) blocks of 16 rows (two when heads x rows exceed 16); a partial slot holds
// 16 x blocks rows.
int mq_row_blocks(int G, int q_len);
int mq_heads_per_pass(int G, int q_len);
hipError_t launch_attn_mq(const Shape& s, const LayerView& lv, const Scratch& sc, int q_len, const void* q,
                          const void* k_new, const void* v_new, const SeqMask& mask, const InlineLens& lens,
                          int keys_per_group, int n_groups, hipStream_t st, const KernelTimer* tm = nullptr);
hipError_t attn_mq_groups_per_cu(const Shape& s, int* out);
// `narrow`: the launch's flattened key axis is shorter than 2^31 positions.
hipError_t launch_finish_mq(const Shape& s, const LayerView& lv, const Scratch& sc, int q_len, void* out,
                            const SeqMask& mask, const InlineLens& lens, int max_nd_eff, int keys_per_group,
                            bool narrow, hipStream_t st, const KernelTimer* tm = nullptr);

// Compaction of the slots marked in LayerView::dead (plus the pending selection) for the masked
// sequences: survivors move down in order, the bitmaps are cleared, nd becomes the live count.
hipError_t launch_compact_holes(const Shape& s, const LayerView& lv, const Scratch& sc, const SeqMask& mask,
                                hipStream_t st, const KernelTimer* tm = nullptr);

// One-token eviction of the sequences whose evict_key is set, all of which hold budget + 1 tokens:
// the selection was made by the finishing kernel, this only closes the gap.
hipError_t launch_evict_one(const Shape& s, const LayerView& lv, const Scratch& sc, const SeqMask& mask,
                            hipStream_t st, const KernelTimer* tm = nullptr);

// k/v projection + rotary encoding of the appended token, written into slot nd[b] of the decode
// pool (bf16 only; hidden a multiple of 256).
// `part`: scratch of project_ksplit(hidden) * B * 2 * Hkv * D floats.
int project_ksplit(int hidden);
hipError_t launch_project_append(const Shape& s, const LayerView& lv, const SeqMask& mask, const void* x,
                                 const void* wk, const void* wv, const int32_t* rope_pos, float* part,
                                 int hidden, float rope_theta, hipStream_t st, const KernelTimer* tm = nullptr);

hipError_t configure_kernels();

// Virtual positions of a unit on the flattened key axis beside its M + n1 keys: piece_pad in front
// of the keys, tail_pad behind them.
__host__ __device__ inline int unit_extra(const Shape& s) { return s.piece_pad + s.tail_pad; }

inline int head_lanes(int G) { return G == 1 ? 1 : G == 2 ? 2 : G <= 4 ? 4 : 8; }

}  // namespace mkv
