// Host-side pieces shared by the operator files: context, error reporting, shape resolution.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "../../include/tilelink_mi355.h"
#include "tl_ag_producer.h"
#include "tl_device.h"
#include "tl_gemm_tile.h"
#include "tl_rs_consumer.h"

struct tl_ctx {
  tl_config cfg;
  int device;
  int num_cus;
};

namespace tl {

void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);

#define TL_HIP(expr)                                                                          \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess) return tl::fail(TL_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// Tile shapes the GEMM kernels are instantiated for.
enum TileVariant { TILE_256x256 = 0, TILE_256x224 = 1, TILE_128x128 = 2, TILE_VARIANTS = 3 };

// Everything the host decides before a dense (AG+GEMM or GEMM+RS) launch.
struct Resolved {
  int variant, tile_m, tile_n;
  int nbm, nbn, n_tiles;
  int G, n_comm;
  int Tm_p, Tn_p;        // producer / reduce tile
  int n_ptm, n_ptn;      // producer or reduce tiles along rows / columns
  int rows_per_rank, rows_per_channel;
  int expected;          // producer tiles per channel (AG) ; not used by RS
  int threads, lds_bytes;
  int first_block;       // rotation of row blocks in the compute order
  int group_m;           // row blocks per group of the compute order
  int k_chunks;          // AG+GEMM: flags per channel along K (1 = one flag per channel)
  int arrival_bpr;       // AG+GEMM under TL_ORDER_ARRIVAL: row blocks per rank (0 = another order)
};

// paired_columns: the tile's 32-wide column blocks must come in pairs (gated epilogue): no 224-wide tile, N % 64 == 0
int resolve_dense(const tl_ctx* ctx, int op, int M, int N, int K, Resolved* r, bool paired_columns = false);

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

static const int kTileM[TILE_VARIANTS] = {256, 256, 128};
static const int kTileN[TILE_VARIANTS] = {256, 224, 128};
typedef TileCfg<256, 256, 2, 4, 32, 4> Cfg256x256;
typedef TileCfg<256, 224, 8, 1, 32, 4> Cfg256x224;
typedef TileCfg<128, 128, 2, 2, 32, 4> Cfg128x128;
// Row tiles of a grouped GEMM with at most 64 rows (the rest of an expert's rows): their time is the streaming of the
// expert's weight block, which is bound by the bytes in flight -- seven stages of 4 + 16 KiB instead of four of 16 + 16.
typedef TileCfg<64, 256, 2, 4, 32, 7> Cfg64x256;
static const int kThreads[TILE_VARIANTS] = {Cfg256x256::NTHREADS, Cfg256x224::NTHREADS, Cfg128x128::NTHREADS};
static const int kLds[TILE_VARIANTS] = {Cfg256x256::LDS_BYTES, Cfg256x224::LDS_BYTES, Cfg128x128::LDS_BYTES};

inline bool aligned128(const void* p) { return ((uintptr_t)p & 127) == 0; }

inline WaitCtl make_ctl(const tl_ctx* ctx, void* workspace) {
  WaitCtl c;
  c.status = (int*)workspace;
  c.timeout = (unsigned long long)ctx->cfg.spin_timeout_us * 100ull;  // 100 MHz wall clock
  c.strict = 0;
  return c;
}

// Launches a kernel that uses Cfg::LDS_BYTES of dynamic LDS.
template <class Cfg, class P>
inline int launch_fused(void (*kernel)(const P), const P& p, int grid, hipStream_t stream, int lds_bytes = Cfg::LDS_BYTES) {
  TL_HIP(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(Cfg::NTHREADS), lds_bytes, stream, p);
  TL_HIP(hipGetLastError());
  return TL_OK;
}

// Fills the AllGather side of a call (wait_target is left to the caller: it depends on the binding).
inline void fill_ag_producer(const tl_ctx* ctx, AgProducer* p, const void* const* shards, void* gathered, int ld, int Tm_p, int Tn_p,
                             int n_ptm, int n_ptn, int rows_per_rank, int rows_per_channel, unsigned* flags, unsigned epoch,
                             void* workspace) {
  const tl_config& cfg = ctx->cfg;
  for (int q = 0; q < cfg.world_size; q++) p->shards[q] = (const bf16_t*)shards[q];
  p->gathered = (bf16_t*)gathered;
  p->ld = ld;
  p->R = cfg.world_size;
  p->rank = cfg.rank;
  p->Tm_p = Tm_p; p->Tn_p = Tn_p; p->n_ptm = n_ptm; p->n_ptn = n_ptn;
  p->first_src = (cfg.rank + 1) % cfg.world_size;
  p->n_ptm_all = n_ptm;
  p->rows_per_rank = rows_per_rank;
  p->rows_per_channel = rows_per_channel;
  p->local_in_place = (const bf16_t*)shards[cfg.rank] == (const bf16_t*)gathered + (size_t)cfg.rank * rows_per_rank * ld;
  p->k_chunks = 1;
  p->n_out = 0;
  p->pushed = nullptr;
  // simulated links: all source ranks deliver side by side, each at link_gbps
  p->interleave = (cfg.link_gbps > 0 && n_ptm / (rows_per_rank / Tm_p) > 1) ? 1 : 0;
  p->pace_q8 = cfg.link_gbps > 0 ? (unsigned)((double)Tm_p * Tn_p * sizeof(bf16_t) * 256.0 / (cfg.link_gbps * 10.0) + 0.5) : 0;
  p->pace_word = (unsigned long long*)((char*)workspace + 16);
  p->epoch = epoch;
  p->flags = flags;
  p->ticket = (unsigned*)workspace + 1;  // word 0 of the workspace is the status word
  p->ticket_end = epoch * (unsigned)(n_ptm * n_ptn);
  p->ctl = make_ctl(ctx, workspace);
  // a channel is a block of whole rows: its edges fall on 128-byte lines if the pitch and the base do
  p->ctl.strict = (ld % 64 == 0 && aligned128(gathered)) ? 0 : 1;
}

// Fills the ReduceScatter side of a call.  Flags: ready[ncm*ncn] | arrived[R*tiles_per_seg] | pushed[R*tiles_per_seg].
inline void fill_rs_side(const tl_ctx* ctx, RsSide* p, void* partial, const void* const* peer_recv, void* const* peer_push, void* out,
                         int M, int N, int tile_m, int tile_n, int Tm_r, int Tn_r, unsigned* flags, unsigned epoch, void* workspace) {
  const tl_config& cfg = ctx->cfg;
  const int R = cfg.world_size;
  p->partial = (bf16_t*)partial;
  p->out = (bf16_t*)out;
  for (int q = 0; q < R; q++) {
    p->peer_recv[q] = (const bf16_t*)peer_recv[q];
    p->peer_push[q] = (bf16_t*)peer_push[q];
  }
  p->M = M; p->N = N; p->R = R; p->rank = cfg.rank;
  p->tile_m = tile_m; p->tile_n = tile_n;
  p->Tm_r = Tm_r; p->Tn_r = Tn_r; p->ncm = M / Tm_r; p->ncn = N / Tn_r;
  p->direct = cfg.rs_direct_push == 2 ? 2 : (cfg.rs_direct_push ? 1 : 0);
  p->seg_rows = M / R;
  p->fast_rows = (long)(M / R) * N * 2 < (1L << 32) ? 1 : 0;
  p->tiles_per_seg = (p->seg_rows / Tm_r) * p->ncn;
  p->rs_first_block = 0;
  p->do_wait = 1;
  p->epoch = epoch;
  p->ready = flags;
  p->arrived = flags + (size_t)p->ncm * p->ncn;
  p->pushed = p->arrived + (size_t)R * p->tiles_per_seg;
  p->ctl = make_ctl(ctx, workspace);
  // own-segment reduce tiles are handed out in row slices of about 32 rows; no item queue unless the caller sets one up
  p->slices = Tm_r >= 64 ? (Tm_r / 32 < 8 ? Tm_r / 32 : 8) : 1;
  p->queue = nullptr;
  p->queue_end = 0;
  p->others_done = 0;
  // reduce tiles whose edges do not fall on 128-byte lines share cache lines with their neighbours
  bool aligned = N % 64 == 0 && Tn_r % 64 == 0 && aligned128(partial);
  for (int q = 0; q < R; q++)
    if (q != cfg.rank && !aligned128(peer_recv[q])) aligned = false;
  p->ctl.strict = aligned ? 0 : 1;
}

int launch_peers_arrive(const RsSide& rs, hipStream_t s);

// The reduce side as a kernel of its own takes its work items from a queue (word 1 of the workspace, which grows by the
// items of every call: zeroed with the flags, one call at a time).  Call once p->ring is final.
inline void use_rs_queue(RsSide* p, void* workspace, unsigned epoch) {
  // with direct push a reduce tile of another segment that lies inside one producer tile is announced by its producer
  p->others_done = (p->direct && !p->ring && p->do_wait && p->tile_m % p->Tm_r == 0 && p->tile_n % p->Tn_r == 0 && p->N % p->Tn_r == 0) ? 1 : 0;
  p->queue = (unsigned*)workspace + 1;
  p->queue_end = epoch * (unsigned)rs_item_count(*p);
}

inline int check_ctx(const tl_ctx* ctx) {
  if (!ctx) return fail(TL_ERR_INVALID_ARG, "context is null");
  return TL_OK;
}

// For the calls that enqueue GPU work: a context made by tl_ctx_create_host serves the host-side queries only.
inline int check_op_ctx(const tl_ctx* ctx) {
  if (!ctx) return fail(TL_ERR_INVALID_ARG, "context is null");
  if (ctx->device < 0) return fail(TL_ERR_INVALID_ARG, "this context was made by tl_ctx_create_host: it answers queries but cannot launch work");
  return TL_OK;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace tl
