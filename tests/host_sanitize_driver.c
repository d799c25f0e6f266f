/* Walks the library's host-side logic (shape rules, geometry queries, schedule dumps, argument checks) through a context
 * made by tl_ctx_create_host -- no GPU, no HIP call -- for a build whose host code carries AddressSanitizer and
 * UndefinedBehaviorSanitizer.  Prints "host_sanitize_driver ok <calls>" and exits 0 when every call returned what it
 * should; the sanitizers abort the program on their own findings. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "tilelink_mi355.h"

static int calls = 0, bad = 0;
#define EXPECT(cond) do { calls++; if (!(cond)) { bad++; fprintf(stderr, "line %d: %s failed (%s)\n", __LINE__, #cond, tl_last_error()); } } while (0)

static tl_ctx* make(int R, int rank, int C, int mode, int order, int swz, int gm, int tm, int tn, int ctm, int ctn, int kc, int link) {
  tl_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.world_size = R; cfg.rank = rank; cfg.channels_per_rank = C; cfg.comm_mode = mode; cfg.tile_order = order; cfg.xcd_swizzle = swz;
  cfg.group_m = gm; cfg.tile_m = tm; cfg.tile_n = tn; cfg.comm_tile_m = ctm; cfg.comm_tile_n = ctn; cfg.ag_k_chunks = kc; cfg.link_gbps = link;
  cfg.rs_direct_push = 1;
  tl_ctx* ctx = NULL;
  if (tl_ctx_create_host(&cfg, 256, &ctx) != TL_OK) return NULL;
  return ctx;
}

static void dump(tl_ctx* ctx, int op, long long M, long long N, long long K) {
  long long dims[3] = {M, N, K};
  size_t n = 0, ws = 0, nf = 0;
  int info[14];
  int e = tl_query_workspace(ctx, op, dims, &ws, &nf);
  calls++;
  if (e != TL_OK) return;   /* a shape the mapping refuses: every later call refuses it too */
  EXPECT(tl_resolve(ctx, op, dims, info) == TL_OK);
  EXPECT(tl_dump_schedule(ctx, op, dims, NULL, 0, &n) == TL_ERR_WORKSPACE_TOO_SMALL && n > 0);
  int* buf = (int*)malloc(n * sizeof(int));   /* exactly the size asked for: a write past it is the sanitizer's to find */
  size_t n2 = 0;
  EXPECT(tl_dump_schedule(ctx, op, dims, buf, n, &n2) == TL_OK && n2 == n);
  EXPECT(tl_dump_schedule(ctx, op, dims, buf, n - 1, &n2) == TL_ERR_WORKSPACE_TOO_SMALL);
  long long seen = 0;
  for (size_t i = 0; i < n; i++) seen += buf[i];
  if (seen == -1) printf("unlikely\n");
  free(buf);
}

int main(void) {
  static const int modes[] = {TL_COMM_NONE, TL_COMM_WAVES, TL_COMM_STREAM, TL_COMM_SIDE_KERNEL, TL_COMM_COPY_ENGINE};
  static const int orders[] = {TL_ORDER_NATURAL, TL_ORDER_RING, TL_ORDER_OWN_FIRST, TL_ORDER_ARRIVAL};
  static const long long shapes[][3] = {{8192, 3584, 8192}, {8192, 8192, 3584}, {2048, 456, 1024}, {256, 512, 512}, {8192, 1376, 4096}, {8192, 4096, 1376},
                                        {1024, 8, 8}, {8192, 3696, 8192}, {512, 264, 72}, {100, 64, 64}, {8192, 3584, 8190}};
  static const int tiles[][2] = {{0, 0}, {256, 256}, {256, 224}, {128, 128}};
  for (unsigned m = 0; m < sizeof modes / sizeof *modes; m++)
    for (unsigned o = 0; o < sizeof orders / sizeof *orders; o++)
      for (unsigned t = 0; t < sizeof tiles / sizeof *tiles; t++)
        for (int rank = 0; rank < 8; rank += 3) {
          tl_ctx* ctx = make(8, rank, 1 + (int)(o % 2) * 3, modes[m], orders[o], (int)(t % 2), (int)t * 3, tiles[t][0], tiles[t][1], 0, 0, (int)(o == 3) * 4, (int)(o == 3) * 153);
          EXPECT(ctx != NULL);
          if (!ctx) continue;
          for (unsigned s = 0; s < sizeof shapes / sizeof *shapes; s++) {
            dump(ctx, TL_OP_AG_GEMM, shapes[s][0], shapes[s][1], shapes[s][2]);
            dump(ctx, TL_OP_GEMM_RS, shapes[s][0], shapes[s][1], shapes[s][2]);
          }
          int info[8];
          calls++; (void)tl_moe_query(ctx, TL_OP_MOE_AG_GATHER_GEMM, 8192, 4096, 1792, 32, 2, info);
          calls++; (void)tl_moe_query(ctx, TL_OP_MOE_GEMM_SCATTER_RS, 8192, 4096, 1792, 32, 2, info);
          calls++; (void)tl_moe_query(ctx, TL_OP_MOE_GEMM_SCATTER_RS, 8192, 2048, 192, 8, 5, info);
          calls++; (void)tl_attn_query(ctx, 32768, 32, 128, 1, info);
          calls++; (void)tl_attn_query(ctx, 8192, 64, 128, 0, info);
          EXPECT(tl_ctx_destroy(ctx) == TL_OK);
        }
  /* small worlds, reduce tiles that differ from the GEMM tile, producer tiles narrower than a row */
  for (int R = 1; R <= 4; R++) {
    tl_ctx* ctx = make(R, R - 1, 2, TL_COMM_SIDE_KERNEL, TL_ORDER_OWN_FIRST, 1, 0, 0, 0, 64, 512, 0, 0);
    EXPECT(ctx != NULL);
    if (!ctx) continue;
    dump(ctx, TL_OP_AG_GEMM, 2048, 1024, 1024);
    dump(ctx, TL_OP_GEMM_RS, 2048, 1024, 1024);
    EXPECT(tl_ctx_destroy(ctx) == TL_OK);
  }
  /* what must be refused */
  tl_config cfg;
  memset(&cfg, 0, sizeof cfg);
  tl_ctx* ctx = NULL;
  EXPECT(tl_ctx_create_host(&cfg, 256, &ctx) == TL_ERR_INVALID_ARG);           /* world_size 0 */
  cfg.world_size = 8; cfg.rank = 8; cfg.channels_per_rank = 1;
  EXPECT(tl_ctx_create_host(&cfg, 256, &ctx) == TL_ERR_INVALID_ARG);           /* rank outside the world */
  cfg.rank = 0; cfg.comm_mode = 99;
  EXPECT(tl_ctx_create_host(&cfg, 256, &ctx) == TL_ERR_INVALID_ARG);
  cfg.comm_mode = TL_COMM_WAVES;
  EXPECT(tl_ctx_create_host(NULL, 256, &ctx) == TL_ERR_INVALID_ARG);
  EXPECT(tl_ctx_create_host(&cfg, 256, NULL) == TL_ERR_INVALID_ARG);
  cfg.channels_per_rank = 16;                                                   /* 128 channels: more than the wait mask holds */
  EXPECT(tl_ctx_create_host(&cfg, 256, &ctx) == TL_OK);
  long long dims[3] = {8192, 512, 512};
  size_t ws = 0, nf = 0;
  EXPECT(tl_query_workspace(ctx, TL_OP_AG_GEMM, dims, &ws, &nf) == TL_ERR_UNSUPPORTED_SHAPE);
  EXPECT(tl_query_workspace(ctx, TL_OP_AG_GEMM, NULL, &ws, &nf) == TL_ERR_INVALID_ARG);
  EXPECT(tl_query_workspace(ctx, 12345, dims, &ws, &nf) != TL_OK);
  /* a host-only context launches nothing */
  void* fake[8] = {0};
  EXPECT(tl_ag_gemm(ctx, (const void* const*)fake, fake, fake, fake, 8192, 512, 512, (unsigned*)fake, 1, fake, 256, NULL, NULL) != TL_OK);
  EXPECT(tl_check_status(ctx, fake) != TL_OK);
  long long clk[2];
  EXPECT(tl_read_clocks(ctx, fake, clk) != TL_OK);
  EXPECT(tl_ctx_destroy(ctx) == TL_OK);
  EXPECT(tl_version() != NULL && tl_last_error() != NULL);
  if (bad) { fprintf(stderr, "%d of %d checks failed\n", bad, calls); return 1; }
  printf("host_sanitize_driver ok %d\n", calls);
  return 0;
}
