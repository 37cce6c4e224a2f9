/* A decode loop through the C ABI from plain C99, with device memory from hipMalloc and no Python
 * or PyTorch in the process: the library links only the HIP runtime, and this is what a caller
 * written in C sees.  Built by the package's build step, run by tests/test_gpu_c_abi.py, which
 * writes the input file from the seeded generators and holds the output file against the CPU
 * oracle.
 *
 *   abi_gpu_driver <input file> <output file>
 *
 * Input:  int32 header {batch, n_q_heads, n_kv_heads, head_dim, bf16 (0/1), decode_budget,
 *         evict_trigger, recent_window, steps, static_scratch (0/1)}, float alpha, int32 prefill
 *         lengths [batch]; then per sequence the prompt's K and V, float32 [M_s][n_kv_heads][head_dim]
 *         each; then per step q [batch][n_q_heads][head_dim], k_new and v_new
 *         [batch][n_kv_heads][head_dim], float32.  With bf16 = 1 every value is exactly
 *         representable in bfloat16 and is handed to the library as its upper 16 bits.
 * Output: per step Att [batch][n_q_heads][head_dim] as float32 and the decode pool sizes int32
 *         [batch]; at the end per sequence int32 n, float scores [n], int32 positions [n].
 * Exit status 0 and "ok" on stdout; any failing call prints its message and exits 1. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "mkv.h"

#define HIP_OK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
  printf("line %d: %s: %s\n", __LINE__, #call, hipGetErrorString(e_)); exit(1); } } while (0)
#define MKV_OK_(ctx, call) do { int rc_ = (call); if (rc_ != MKV_OK) { \
  printf("line %d: %s: %d %s\n", __LINE__, #call, rc_, mkv_last_error(ctx)); exit(1); } } while (0)

static void read_exact(void* dst, size_t bytes, FILE* f) {
  if (bytes && fread(dst, 1, bytes, f) != bytes) { printf("input file too short\n"); exit(1); }
}

/* float32 values -> the storage dtype's bytes (bf16: upper halves; the values are representable) */
static void to_storage(const float* src, void* dst, size_t n, int bf16) {
  if (!bf16) { memcpy(dst, src, n * 4); return; }
  uint16_t* d = (uint16_t*)dst;
  for (size_t i = 0; i < n; ++i) {
    uint32_t u;
    memcpy(&u, &src[i], 4);
    if (u & 0xFFFFu) { printf("value %zu is not representable in bfloat16\n", i); exit(1); }
    d[i] = (uint16_t)(u >> 16);
  }
}

static void from_storage(const void* src, float* dst, size_t n, int bf16) {
  if (!bf16) { memcpy(dst, src, n * 4); return; }
  const uint16_t* s = (const uint16_t*)src;
  for (size_t i = 0; i < n; ++i) {
    uint32_t u = (uint32_t)s[i] << 16;
    memcpy(&dst[i], &u, 4);
  }
}

int main(int argc, char** argv) {
  if (argc != 3) { printf("usage: %s <input> <output>\n", argv[0]); return 1; }
  FILE* in = fopen(argv[1], "rb");
  FILE* out = fopen(argv[2], "wb");
  if (!in || !out) { printf("cannot open the files\n"); return 1; }
  int32_t h[10];
  float alpha;
  read_exact(h, sizeof h, in);
  read_exact(&alpha, 4, in);
  const int B = h[0], H = h[1], Hkv = h[2], D = h[3], bf16 = h[4], budget = h[5], trigger = h[6], W = h[7],
            steps = h[8], use_static = h[9];
  if (B < 1 || B > 64 || H < 1 || Hkv < 1 || (D != 64 && D != 128) || steps < 0) { printf("bad header\n"); return 1; }
  int32_t* M = (int32_t*)malloc((size_t)B * 4);
  read_exact(M, (size_t)B * 4, in);
  int max_m = 0;
  for (int b = 0; b < B; ++b) {
    if (M[b] < 0 || M[b] > (1 << 20)) { printf("bad prefill length\n"); return 1; }
    if (M[b] > max_m) max_m = M[b];
  }
  const size_t es = bf16 ? 2 : 4;

  HIP_OK(hipSetDevice(0));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));

  mkv_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = 1; cfg.batch = B; cfg.n_q_heads = H; cfg.n_kv_heads = Hkv; cfg.head_dim = D;
  cfg.dtype = bf16 ? MKV_BF16 : MKV_F32;
  cfg.max_prefill = max_m; cfg.decode_budget = budget; cfg.evict_trigger = trigger; cfg.recent_window = W;
  cfg.alpha = alpha;
  cfg.stream = (void*)stream;                  /* arena NULL: the library allocates its own memory */
  mkv_ctx* ctx = NULL;
  MKV_OK_(NULL, mkv_create(&cfg, &ctx));
  if (mkv_required_bytes(&cfg) == 0) { printf("mkv_required_bytes is 0 for a configuration that was accepted\n"); return 1; }

  /* prompt */
  for (int b = 0; b < B; ++b) {
    const size_t n = (size_t)M[b] * Hkv * D;
    if (!n) continue;
    float* hk = (float*)malloc(n * 4);
    float* hv = (float*)malloc(n * 4);
    void* sk = malloc(n * es);
    void* sv = malloc(n * es);
    read_exact(hk, n * 4, in);
    read_exact(hv, n * 4, in);
    to_storage(hk, sk, n, bf16);
    to_storage(hv, sv, n, bf16);
    void *dk, *dv;
    HIP_OK(hipMalloc(&dk, n * es));
    HIP_OK(hipMalloc(&dv, n * es));
    HIP_OK(hipMemcpy(dk, sk, n * es, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dv, sv, n * es, hipMemcpyHostToDevice));
    /* in two parts: the second append lands behind the first */
    const int first = M[b] / 3;
    MKV_OK_(ctx, mkv_prefill_append(ctx, 0, b, dk, dv, first));
    MKV_OK_(ctx, mkv_prefill_append(ctx, 0, b, (char*)dk + (size_t)first * Hkv * D * es,
                                    (char*)dv + (size_t)first * Hkv * D * es, M[b] - first));
    HIP_OK(hipStreamSynchronize(stream));      /* the library copies the rows on its stream */
    HIP_OK(hipFree(dk));
    HIP_OK(hipFree(dv));
    free(hk); free(hv); free(sk); free(sv);
  }

  /* decode loop */
  const size_t nq = (size_t)B * H * D, nkv = (size_t)B * Hkv * D;
  float* hq = (float*)malloc(nq * 4);
  float* hkn = (float*)malloc(nkv * 4);
  float* hvn = (float*)malloc(nkv * 4);
  float* ho = (float*)malloc(nq * 4);
  void* sq = malloc(nq * es);
  void* skn = malloc(nkv * es);
  void* svn = malloc(nkv * es);
  void* so = malloc(nq * es);
  void *dq, *dkn, *dvn, *dout;
  HIP_OK(hipMalloc(&dq, nq * es));
  HIP_OK(hipMalloc(&dkn, nkv * es));
  HIP_OK(hipMalloc(&dvn, nkv * es));
  HIP_OK(hipMalloc(&dout, nq * es));
  int32_t* lens = (int32_t*)malloc((size_t)B * 4);
  for (int t = 0; t < steps; ++t) {
    read_exact(hq, nq * 4, in);
    read_exact(hkn, nkv * 4, in);
    read_exact(hvn, nkv * 4, in);
    to_storage(hq, sq, nq, bf16);
    to_storage(hkn, skn, nkv, bf16);
    to_storage(hvn, svn, nkv, bf16);
    HIP_OK(hipMemcpyAsync(dq, sq, nq * es, hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(dkn, skn, nkv * es, hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(dvn, svn, nkv * es, hipMemcpyHostToDevice, stream));
    if (use_static) MKV_OK_(ctx, mkv_decode_step_static(ctx, 0, dq, dkn, dvn, dout, NULL));
    else MKV_OK_(ctx, mkv_decode_step(ctx, 0, dq, dkn, dvn, dout, NULL));
    HIP_OK(hipMemcpyAsync(so, dout, nq * es, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    from_storage(so, ho, nq, bf16);
    fwrite(ho, 4, nq, out);
    for (int b = 0; b < B; ++b) {
      int n_pre = -1, n_dec = -1;
      int64_t step = -1;
      MKV_OK_(ctx, mkv_get_lens(ctx, 0, b, &n_pre, &n_dec, &step));
      if (n_pre != M[b] || step != t + 1) { printf("step %d seq %d: lengths %d %lld\n", t, b, n_pre, (long long)step); return 1; }
      lens[b] = n_dec;
    }
    fwrite(lens, 4, (size_t)B, out);
  }

  /* the pools at the end */
  for (int b = 0; b < B; ++b) {
    int n = 0;
    MKV_OK_(ctx, mkv_read_scores(ctx, 0, b, NULL, NULL, 0, &n));
    float* sc = (float*)malloc((size_t)(n > 0 ? n : 1) * 4);
    int32_t* pos = (int32_t*)malloc((size_t)(n > 0 ? n : 1) * 4);
    int n2 = 0;
    MKV_OK_(ctx, mkv_read_scores(ctx, 0, b, sc, pos, n, &n2));
    if (n2 != n) { printf("seq %d: pool size changed between two reads\n", b); return 1; }
    int32_t n32 = n;
    fwrite(&n32, 4, 1, out);
    fwrite(sc, 4, (size_t)n, out);
    fwrite(pos, 4, (size_t)n, out);
    free(sc); free(pos);
  }
  /* a call that must be refused leaves a message and the state as it was */
  if (steps > 0) {
    int n_before = -1, n_after = -1;
    MKV_OK_(ctx, mkv_get_lens(ctx, 0, 0, &n_before, NULL, NULL));
    if (mkv_prefill_append(ctx, 0, 0, dkn, dvn, 1) != MKV_ERR_FROZEN || strlen(mkv_last_error(ctx)) == 0) {
      printf("prefill append after the first decode step was not refused\n");
      return 1;
    }
    MKV_OK_(ctx, mkv_get_lens(ctx, 0, 0, &n_after, NULL, NULL));
    if (n_after != n_before) { printf("a refused call changed the prompt length\n"); return 1; }
  }
  MKV_OK_(NULL, mkv_destroy(ctx));
  HIP_OK(hipFree(dq)); HIP_OK(hipFree(dkn)); HIP_OK(hipFree(dvn)); HIP_OK(hipFree(dout));
  HIP_OK(hipStreamDestroy(stream));
  fclose(in);
  if (fclose(out) != 0) { printf("writing the output failed\n"); return 1; }
  free(hq); free(hkn); free(hvn); free(ho); free(sq); free(skn); free(svn); free(so); free(lens); free(M);
  printf("ok\n");
  return 0;
}
