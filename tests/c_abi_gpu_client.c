/* A plain C client of include/lkv.h that runs the four hot calls on a GPU: device memory comes from the HIP
 * runtime's C interface, nothing from PyTorch.  It reads one small problem from a file, runs
 * lkv_score -> lkv_select -> lkv_compact -> lkv_decode_attn, writes every result to a file (the test compares
 * them with the oracle), and checks that the hot calls refuse bad arguments on a live context before they
 * enqueue anything.  Built and run by tests/test_gpu_c_client.py.
 *
 * Input file (little endian): int32 L, H, Hq, T, kind, hidden, act, per_head, has_b2;
 *   K, V   bf16 [L, H, T, 128];  w1 bf16 [rows, 256] (linear) or [rows, hidden, 256];  b1 fp32 [rows] or [rows, hidden];
 *   w2 fp32 [rows, hidden] and, if has_b2, b2 fp32 [rows] (MLP only);  budgets int32 [L, H];  q bf16 [L, Hq, 128];
 *   rows = L * (per_head ? H : 1).
 * Output file: int64 total;  scores fp32 [L, H, T];  offsets int32 [L H + 1];  idx int32 [total];
 *   kp, vp bf16 [total, 128];  out fp32 [L, Hq, 128];  lse fp32 [L, Hq]. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "lkv.h"

#define CHECK(cond)                                                              \
  do {                                                                           \
    if (!(cond)) {                                                               \
      fprintf(stderr, "line %d: %s (%s)\n", __LINE__, #cond, lkv_last_error(ctx)); \
      return 1;                                                                  \
    }                                                                            \
  } while (0)

static void *read_block(FILE *f, size_t bytes) {
  void *p = malloc(bytes ? bytes : 1);
  if (p != NULL && bytes != 0 && fread(p, 1, bytes, f) != bytes) {
    free(p);
    return NULL;
  }
  return p;
}

static void *to_device(const void *host, size_t bytes) {
  void *d = NULL;
  if (hipMalloc(&d, bytes ? bytes : 16) != hipSuccess) return NULL;
  if (bytes != 0 && hipMemcpy(d, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
  return d;
}

static int write_device(FILE *f, const void *dev, size_t bytes) {
  void *h = malloc(bytes ? bytes : 1);
  int ok = h != NULL && (bytes == 0 || hipMemcpy(h, dev, bytes, hipMemcpyDeviceToHost) == hipSuccess) &&
           fwrite(h, 1, bytes, f) == bytes;
  free(h);
  return ok;
}

int main(int argc, char **argv) {
  lkv_ctx *ctx = NULL;
  int32_t hd[9];
  FILE *in, *outf;
  if (argc != 3) return 2;
  in = fopen(argv[1], "rb");
  if (in == NULL || fread(hd, sizeof(int32_t), 9, in) != 9) return 2;
  {
    const int32_t L = hd[0], H = hd[1], Hq = hd[2], T = hd[3], kind = hd[4], hidden = hd[5], act = hd[6], per_head = hd[7],
                  has_b2 = hd[8];
    const size_t rows = (size_t)L * (per_head ? H : 1), n_seg = (size_t)L * H, d = 128;
    const size_t kv_bytes = n_seg * T * d * 2;
    const size_t w1_bytes = rows * (kind == LKV_SCORER_MLP ? hidden : 1) * 256 * 2;
    const size_t b1_bytes = rows * (kind == LKV_SCORER_MLP ? hidden : 1) * 4;
    const size_t w2_bytes = kind == LKV_SCORER_MLP ? rows * hidden * 4 : 0;
    const size_t b2_bytes = kind == LKV_SCORER_MLP && has_b2 ? rows * 4 : 0;
    void *hK = read_block(in, kv_bytes), *hV = read_block(in, kv_bytes), *hw1 = read_block(in, w1_bytes);
    void *hb1 = read_block(in, b1_bytes), *hw2 = read_block(in, w2_bytes), *hb2 = read_block(in, b2_bytes);
    int32_t *budgets = (int32_t *)read_block(in, n_seg * 4);
    void *hq = read_block(in, (size_t)L * Hq * d * 2);
    int64_t total = 0;
    size_t i, ws_bytes;
    void *dK, *dV, *dq, *dkp, *dvp, *dws;
    float *dscores, *dout, *dlse;
    int32_t *didx, *doff;
    const void *kptr[1], *vptr[1];
    float *sptr[1];
    const float *csptr[1];
    int32_t lens[1];
    lkv_cache cache;
    lkv_scorer scorer;
    const float scale = 1.0f / sqrtf(128.0f);

    if (!hK || !hV || !hw1 || !hb1 || !hw2 || !hb2 || !budgets || !hq) return 2;
    fclose(in);
    for (i = 0; i < n_seg; ++i) total += budgets[i];

    CHECK(lkv_create(&ctx, 0) == LKV_OK);
    dK = to_device(hK, kv_bytes);
    dV = to_device(hV, kv_bytes);
    dq = to_device(hq, (size_t)L * Hq * d * 2);
    CHECK(dK && dV && dq);
    memset(&scorer, 0, sizeof(scorer));
    scorer.kind = kind;
    scorer.act = act;
    scorer.hidden = hidden;
    scorer.per_head = per_head;
    scorer.w1 = to_device(hw1, w1_bytes);
    scorer.b1 = (const float *)to_device(hb1, b1_bytes);
    scorer.w2 = w2_bytes ? (const float *)to_device(hw2, w2_bytes) : NULL;
    scorer.b2 = b2_bytes ? (const float *)to_device(hb2, b2_bytes) : NULL;
    CHECK(scorer.w1 && scorer.b1);
    CHECK(hipMalloc((void **)&dscores, n_seg * T * 4) == hipSuccess);
    CHECK(hipMalloc((void **)&didx, (size_t)(total ? total : 1) * 4) == hipSuccess);
    CHECK(hipMalloc((void **)&doff, (n_seg + 1) * 4) == hipSuccess);
    CHECK(hipMalloc(&dkp, (size_t)(total ? total : 1) * d * 2) == hipSuccess);
    CHECK(hipMalloc(&dvp, (size_t)(total ? total : 1) * d * 2) == hipSuccess);
    CHECK(hipMalloc((void **)&dout, (size_t)L * Hq * d * 4) == hipSuccess);
    CHECK(hipMalloc((void **)&dlse, (size_t)L * Hq * 4) == hipSuccess);
    ws_bytes = lkv_decode_workspace_bytes((int32_t)n_seg, total, Hq, H);
    CHECK(hipMalloc(&dws, ws_bytes ? ws_bytes : 256) == hipSuccess);

    lens[0] = T;
    kptr[0] = dK;
    vptr[0] = dV;
    sptr[0] = dscores;
    csptr[0] = dscores;
    memset(&cache, 0, sizeof(cache));
    cache.n_seq = 1;
    cache.n_layers = L;
    cache.n_kv_heads = H;
    cache.n_q_heads = Hq;
    cache.head_dim = 128;
    cache.seq_len = lens;
    cache.k = kptr;
    cache.v = vptr;

    /* ---- the hot calls refuse bad arguments on a live context, and say why ---- */
    {
      lkv_cache bad = cache;
      lkv_scorer bads = scorer;
      float *mis[1];
      int32_t *too_many = (int32_t *)malloc(n_seg * 4);
      bad.head_dim = 64;
      CHECK(lkv_score(ctx, &bad, &scorer, sptr, NULL) == LKV_ERR_UNSUPPORTED);
      CHECK(strlen(lkv_last_error(ctx)) > 0);
      bad = cache;
      bad.n_q_heads = H + 1;                      /* not a multiple of H (H >= 2 in the test) */
      CHECK(lkv_score(ctx, &bad, &scorer, sptr, NULL) == LKV_ERR_INVALID_ARG);
      mis[0] = (float *)((char *)dscores + 4);    /* not 16-byte aligned */
      CHECK(lkv_score(ctx, &cache, &scorer, mis, NULL) == LKV_ERR_INVALID_ARG);
      if (kind == LKV_SCORER_MLP) {
        bads.hidden = 24;                         /* not a multiple of 16 */
        CHECK(lkv_score(ctx, &cache, &bads, sptr, NULL) == LKV_ERR_UNSUPPORTED);
      }
      bads = scorer;
      bads.w1 = NULL;
      CHECK(lkv_score(ctx, &cache, &bads, sptr, NULL) == LKV_ERR_INVALID_ARG);
      CHECK(too_many != NULL);
      memcpy(too_many, budgets, n_seg * 4);
      too_many[n_seg - 1] = T + 1;                /* a budget above the head's length */
      CHECK(lkv_select(ctx, &cache, csptr, too_many, didx, doff, NULL) == LKV_ERR_INVALID_ARG);
      too_many[n_seg - 1] = -1;
      CHECK(lkv_select(ctx, &cache, csptr, too_many, didx, doff, NULL) == LKV_ERR_INVALID_ARG);
      free(too_many);
      CHECK(lkv_select(ctx, &cache, csptr, budgets, NULL, doff, NULL) == LKV_ERR_INVALID_ARG || total == 0);
      CHECK(lkv_compact(ctx, &cache, didx, doff, total, NULL, dvp, NULL) == LKV_ERR_INVALID_ARG || total == 0);
      CHECK(lkv_decode_attn(ctx, 1, L, H, Hq, 128, dq, dkp, dvp, doff, total, scale, dout, dlse, dws, 0, NULL) ==
                LKV_ERR_WORKSPACE || ws_bytes == 0);
      CHECK(lkv_decode_attn(ctx, 1, L, H, Hq, 128, dq, dkp, dvp, doff, total, scale, dout, dlse, NULL, ws_bytes, NULL) ==
                LKV_ERR_WORKSPACE || ws_bytes == 0);
      CHECK(lkv_decode_attn(ctx, 1, L, H, Hq, 64, dq, dkp, dvp, doff, total, scale, dout, dlse, dws, ws_bytes, NULL) ==
            LKV_ERR_UNSUPPORTED);
      CHECK(lkv_decode_attn(ctx, 1, L, H, Hq, 128, NULL, dkp, dvp, doff, total, scale, dout, dlse, dws, ws_bytes, NULL) ==
            LKV_ERR_INVALID_ARG);
    }

    /* ---- the path itself, on the default stream ---- */
    CHECK(lkv_score(ctx, &cache, &scorer, sptr, NULL) == LKV_OK);
    CHECK(lkv_select(ctx, &cache, csptr, budgets, didx, doff, NULL) == LKV_OK);
    CHECK(lkv_compact(ctx, &cache, didx, doff, total, dkp, dvp, NULL) == LKV_OK);
    CHECK(lkv_decode_attn(ctx, 1, L, H, Hq, 128, dq, dkp, dvp, doff, total, scale, dout, dlse, dws, ws_bytes, NULL) == LKV_OK);
    CHECK(hipDeviceSynchronize() == hipSuccess);

    outf = fopen(argv[2], "wb");
    CHECK(outf != NULL);
    CHECK(fwrite(&total, sizeof(total), 1, outf) == 1);
    CHECK(write_device(outf, dscores, n_seg * T * 4));
    CHECK(write_device(outf, doff, (n_seg + 1) * 4));
    CHECK(write_device(outf, didx, (size_t)total * 4));
    CHECK(write_device(outf, dkp, (size_t)total * d * 2));
    CHECK(write_device(outf, dvp, (size_t)total * d * 2));
    CHECK(write_device(outf, dout, (size_t)L * Hq * d * 4));
    CHECK(write_device(outf, dlse, (size_t)L * Hq * 4));
    CHECK(fclose(outf) == 0);
    lkv_destroy(ctx);
  }
  puts("c gpu client ok");
  return 0;
}
