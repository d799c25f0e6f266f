// AllGather+GEMM and GEMM+ReduceScatter: fused persistent kernels, their producers/consumers,
// host-side validation, mapping tables and launches.  gfx950 only.
#include "tl_ag_producer.h"
#include "tl_gemm_tile.h"
#include "tl_host.h"
#include "tl_rs_consumer.h"

#include <mutex>

namespace tl {

// ======================================================================================
// Kernel parameters
// ======================================================================================
struct AgGemmParams {
  AgProducer prod;      // gathered A: shards, buffer, producer tiles, channel flags, ticket queue
  const bf16_t* b;
  bf16_t* c;            // [M, N], or [M, N/2] with an activation
  int M, N, K;
  int act;              // 0, or ACT_*: B holds gate and up columns, the output is act(gate) * up
  Sched sched;
  int n_comm;           // producer workgroups at the front of the grid (0: none in this launch)
  int do_compute;       // 0: producers only
  int do_wait;          // 0: no wait, 1: wait on channel flags and help the producers, 2: wait only
};

struct GemmRsParams {
  RsSide rs;            // partial product, peers, output, reduce tiles and their counters
  const bf16_t* a;
  const bf16_t* b;
  int K;
  Sched sched;
  int n_comm, do_compute, do_notify;
};

// consumer_tile_wait inside the K loop, for AllGather channels that arrive in chunks along K: K step ks opens chunk
// ks / steps_per_chunk; one wave polls the flags of that chunk for every channel the tile's rows touch while the
// other waves go on to the barrier the K loop holds anyway.  The first chunk is waited for before the tile starts.
struct ChunkWait {
  static constexpr bool ENABLED = true;
  unsigned* flags;
  int k_chunks, steps_per_chunk, clo, chi;
  unsigned target;
  WaitCtl ctl;
  __device__ __forceinline__ bool starts(int ks) const { return ks % steps_per_chunk == 0; }
  __device__ __forceinline__ void wait(int ks) const {
    if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) == 0) {   // wave 0, a uniform branch: the K loop holds barriers
      const int kc = ks / steps_per_chunk;
      for (int ch = clo; ch <= chi; ch++) wave_tile_wait(flags + ch * k_chunks + kc, target, ctl, ch * k_chunks + kc);
    }
  }
  __device__ __forceinline__ void acquire() const { acquire_after_wait(ctl); }
};

template <class Cfg, bool GATED = false>
__global__ void __launch_bounds__(Cfg::NTHREADS) ag_gemm_kernel(const AgGemmParams p) {
  typedef typename std::conditional<GATED, GatedRows, DenseRows>::type Out;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int s_ticket;
  const int tid = threadIdx.x;
  if ((int)blockIdx.x < p.n_comm) {
    ag_producer(p.prod, tid, Cfg::NTHREADS, &s_ticket);
    return;
  }
  if (!p.do_compute) return;
  __builtin_amdgcn_s_setprio(TL_COMPUTE_WAVE_PRIO);  // matrix waves go first when they share a SIMD with communication waves
  const int w = blockIdx.x - p.n_comm;
  const int M_per_channel = p.prod.rows_per_channel;
  const ClockSample cs0 = clock_sample_begin(w);
  for (int pos = w; pos < p.sched.n_tiles; pos += p.sched.G) {
    int tile = sched_tile(p.sched, pos);
    int bm = tile / p.sched.nbn, bn = tile - bm * p.sched.nbn;
    int row_lo = bm * Cfg::BM, col_lo = bn * Cfg::BN;
    int rows = min(Cfg::BM, p.M - row_lo), cols = min(Cfg::BN, p.N - col_lo);
    // consumer_tile_wait: every channel whose rows the tile touches
    const int clo = row_lo / M_per_channel, chi = (row_lo + rows - 1) / M_per_channel;
    if (p.do_wait == 1) {
      unsigned long long mask = ((chi - clo + 1 >= 64) ? ~0ull : ((1ull << (chi - clo + 1)) - 1)) << clo;
      consumer_wait_or_produce<8>(p.prod, mask, tid, Cfg::NTHREADS, &s_ticket);
    } else if (p.do_wait == 2) {
      // flags raised by somebody else (no ticket queue): plain wait
      if (tid == 0)
        for (int ch = clo; ch <= chi; ch++) tile_wait(p.prod.flags + ch * p.prod.k_chunks, p.prod.wait_target, p.prod.ctl, ch * p.prod.k_chunks);
      __syncthreads();
    }
    Out out;
    if constexpr (GATED) out = Out{p.c + (long)row_lo * (p.N / 2) + col_lo / 2, p.N / 2, p.act};
    else out = Out{p.c + (long)row_lo * p.N + col_lo, p.N};
    if (p.prod.k_chunks > 1 && p.do_wait) {
      gemm_tile<Cfg>(p.prod.gathered + (long)row_lo * p.K, p.K, nullptr, 1, p.b + col_lo, p.N, out, rows, cols, p.K, smem,
                     ChunkWait{p.prod.flags, p.prod.k_chunks, p.K / Cfg::BK / p.prod.k_chunks, clo, chi, p.prod.wait_target, p.prod.ctl});
    } else {
      gemm_tile<Cfg>(p.prod.gathered + (long)row_lo * p.K, p.K, nullptr, 1, p.b + col_lo, p.N, out, rows, cols, p.K, smem);
    }
  }
  clock_sample_end(cs0, w, p.prod.ctl.status);
}

// Producer as a kernel of its own (small register/LDS footprint, so it can share compute units
// with resident GEMM workgroups) for the side-stream binding.
__global__ void __launch_bounds__(256) ag_producer_kernel(const AgProducer p) {
  __shared__ int s_ticket;
  ag_producer(p, threadIdx.x, 256, &s_ticket);
}

// rank_notify for copies made by the runtime's copy path: raise `count` consecutive flags.
__global__ void notify_kernel(unsigned* flags, int count, unsigned inc) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) tile_notify(flags + i, inc);
}

// producer_tile_notify of one finished GEMM tile: one add per reduce tile it overlaps -- and, for a reduce tile of another
// rank's segment that this tile alone fills, the announcement to its owner (peer_tile_notify) right with it.  The tile's
// rows were stored written-through to device scope (PushRows), so "released" means no more than: every wave has seen its
// stores complete and the workgroup has met at a barrier since; the caller guarantees both (gemm_tile's hook, or an
// explicit wait after the last tile).  Deferring the notification into the next tile's prologue hides that wait behind
// the latency of the next tile's first loads: a release fence at device scope right after the epilogue cost 4-5 us per tile.
struct TileNotify {
  const RsSide* rs;
  bool have;          // false: nothing pending
  int row_lo, col_lo, rows, cols;
  __device__ __forceinline__ bool pending() const { return have; }
  __device__ __forceinline__ void run() const {
    const RsSide& r = *rs;
    const int cm_lo = row_lo / r.Tm_r, cm_hi = (row_lo + rows - 1) / r.Tm_r;
    const int cn_lo = col_lo / r.Tn_r, cn_hi = (col_lo + cols - 1) / r.Tn_r;
    const int ncols = cn_hi - cn_lo + 1, cnt = (cm_hi - cm_lo + 1) * ncols;
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
      const int cm = cm_lo + i / ncols, cn = cn_lo + i % ncols;
      __hip_atomic_fetch_add(r.ready + cm * r.ncn + cn, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const int r_lo = cm * r.Tm_r, c_lo = cn * r.Tn_r;
      const int r_n = min(r.Tm_r, r.M - r_lo), c_n = min(r.Tn_r, r.N - c_lo);
      if (producer_notifies_peer(r, r_lo, r_n, c_lo, c_n)) {
        const int dest = r_lo / r.seg_rows;
        const int local = (cm - dest * (r.seg_rows / r.Tm_r)) * r.ncn + cn;
        __hip_atomic_fetch_add(r.pushed + dest * r.tiles_per_seg + local, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
};

template <class Cfg>
__global__ void __launch_bounds__(Cfg::NTHREADS) gemm_rs_kernel(const GemmRsParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x;
  if ((int)blockIdx.x < p.n_comm) {
    rs_consumer(p.rs, blockIdx.x, p.n_comm, tid, Cfg::NTHREADS);
    return;
  }
  if (!p.do_compute) return;
  __builtin_amdgcn_s_setprio(TL_COMPUTE_WAVE_PRIO);  // matrix waves go first when they share a SIMD with communication waves
  const int w = blockIdx.x - p.n_comm;
  const RsSide& rs = p.rs;
  const ClockSample cs0 = clock_sample_begin(w);
  // the 224-wide tile has no register left for the state a deferred notification carries from tile to tile
  constexpr bool DEFER = Cfg::BN != 224;
  bool have = false;            // the previous tile of this workgroup awaits its notification
  int p_row = 0, p_col = 0, p_rows = 0, p_cols = 0;
  for (int pos = w; pos < p.sched.n_tiles; pos += p.sched.G) {
    int tile = sched_tile(p.sched, pos);
    int bm = tile / p.sched.nbn, bn = tile - bm * p.sched.nbn;
    int row_lo = bm * Cfg::BM, col_lo = bn * Cfg::BN;
    int rows = min(Cfg::BM, rs.M - row_lo), cols = min(Cfg::BN, rs.N - col_lo);
    if (rs.direct == 2 && p.do_notify && row_lo < (rs.rank + 1) * rs.seg_rows && row_lo + rows > rs.rank * rs.seg_rows) {
      // the tile holds rows of the own segment, which its epilogue reduces: peer_tile_wait for every peer's
      // contribution to the reduce tiles of the own segment it covers
      if (tid == 0) {
        const int own_lo = max(row_lo, rs.rank * rs.seg_rows), own_hi = min(row_lo + rows, (rs.rank + 1) * rs.seg_rows);
        const int cm_per_seg = rs.seg_rows / rs.Tm_r;
        for (int cm = own_lo / rs.Tm_r; cm <= (own_hi - 1) / rs.Tm_r; cm++)
          for (int cn = col_lo / rs.Tn_r; cn <= (col_lo + cols - 1) / rs.Tn_r; cn++) {
            const int local = (cm - rs.rank * cm_per_seg) * rs.ncn + cn;
            for (int q = 0; q < rs.R; q++)
              if (q != rs.rank) tile_wait(rs.arrived + q * rs.tiles_per_seg + local, rs.epoch, rs.ctl, rs.ncm * rs.ncn + q * rs.tiles_per_seg + local);
          }
      }
      __syncthreads();
    }
    if constexpr (DEFER) {
      // producer_tile_notify of the PREVIOUS tile happens inside this tile's prologue, once its stores are known complete
      gemm_tile<Cfg>(p.a + (long)row_lo * p.K, p.K, nullptr, 1, p.b + col_lo, rs.N, PushRowsT<true>{&rs, row_lo, col_lo}, rows, cols, p.K, smem, NoKWait{},
                     TileNotify{&rs, have, p_row, p_col, p_rows, p_cols});
      if (p.do_notify) { have = true; p_row = row_lo; p_col = col_lo; p_rows = rows; p_cols = cols; }
    } else {
      gemm_tile<Cfg>(p.a + (long)row_lo * p.K, p.K, nullptr, 1, p.b + col_lo, rs.N, PushRowsT<false, false>{&rs, row_lo, col_lo}, rows, cols, p.K, smem);
      if (p.do_notify) {
        __syncthreads();                                      // every wave's stores are complete ...
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // ... and written back to where every die sees them
        TileNotify{&rs, true, row_lo, col_lo, rows, cols}.run();
      }
    }
  }
  if (have) {   // the last tile: nothing follows that could hide the wait for its stores
    wait_vmcnt<0>();
    __syncthreads();
    TileNotify{&rs, true, p_row, p_col, p_rows, p_cols}.run();
  }
  clock_sample_end(cs0, w, rs.ctl.status);
}

// Achievable-peak probe: nothing but matrix instructions on register operands -- every compute unit runs one workgroup
// of 8 waves (two per SIMD, as in the tile kernels), each wave `iters` times the 8 MFMAs of one k-slice of its 128x64
// wave tile (4 + 2 operand fragments loaded once from `operands`, 8 accumulators).  What this loop reaches on a given
// operand distribution is what the matrix cores sustain at the clock the chip grants for that data; the first
// workgroup leaves its cycle and wall-clock counts in `clocks`.
__global__ void __launch_bounds__(512) mfma_peak_kernel(const u32x4* __restrict__ operands, float* __restrict__ sink, int iters, long long* clocks) {
  const size_t t = (size_t)blockIdx.x * 512 + threadIdx.x;
  u32x4 fa[4], fb[2];
#pragma unroll
  for (int j = 0; j < 4; j++) fa[j] = operands[t * 6 + j];
#pragma unroll
  for (int j = 0; j < 2; j++) fb[j] = operands[t * 6 + 4 + j];
  floatx16 c[8];
#pragma unroll
  for (int j = 0; j < 8; j++)
#pragma unroll
    for (int e = 0; e < 16; e++) c[j][e] = 0.f;
  const long long c0 = clock64();
  const unsigned long long w0 = wall_clock64();
  for (int i = 0; i < iters; i++) {
#pragma unroll
    for (int m = 0; m < 8; m++)
      c[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fb[m & 1]), __builtin_bit_cast(bf16x8, fa[m >> 1]), c[m], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 8; j++)
#pragma unroll
    for (int e = 0; e < 16; e++) sum += c[j][e];
  sink[t] = sum;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = clock64() - c0;
    clocks[1] = (long long)(wall_clock64() - w0);
  }
}

// Issue probe: what a SIMD issues beside a running matrix instruction.  One slot = one 32x32x16 bf16 MFMA (two
// accumulators in turn; MFMA = 0 leaves it out) followed by MODE's vector instructions, written out so that the compiler
// neither merges nor moves them: 1 = six v_fma_f32, 2 = two v_exp_f32, 3 = v_cvt_pk_bf16_f32 + v_max3_f32,
// 4 = one v_dot2c_f32_bf16, 0 = nothing.  All operands are zero: the chip draws little power, the clock stays at its
// maximum, and time per slot compares across modes in cycles.  The first workgroup leaves its clock sample in `clocks`.
template <int MFMA, int MODE>
__global__ void __launch_bounds__(512) issue_probe_kernel(float* __restrict__ sink, int iters, long long* clocks) {
  floatx16 c0, c1;
#pragma unroll
  for (int e = 0; e < 16; e++) { c0[e] = 0.f; c1[e] = 0.f; }
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; e++) { a[e] = (bf16_t)0.f; b[e] = (bf16_t)0.f; }
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; e++) x[e] = 0.f;
  float k1 = sink[0] * 0.f, k2 = 0.f, acc = 0.f;   // (a value the compiler cannot fold)
  unsigned pk = 0;
  const long long t0 = clock64();
  const unsigned long long w0 = wall_clock64();
  for (int i = 0; i < iters; i++) {
#pragma unroll
    for (int s = 0; s < 8; s++) {
      if constexpr (MFMA != 0) {
        if (s & 1) c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        else c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
      }
      if constexpr (MODE == 1) {
#pragma unroll
        for (int v = 0; v < 6; v++) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[v]) : "v"(k1), "v"(k2));
      } else if constexpr (MODE == 2) {
        asm volatile("v_exp_f32 %0, %1" : "=v"(x[0]) : "v"(x[1]));
        asm volatile("v_exp_f32 %0, %1" : "=v"(x[2]) : "v"(x[3]));
      } else if constexpr (MODE == 3) {
        asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk) : "v"(x[0]), "v"(x[1]));
        asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(x[2]) : "v"(x[3]), "v"(k2));
      } else if constexpr (MODE == 4) {
        asm volatile("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(acc) : "v"(pk), "v"(0x3f803f80u));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const long long t1 = clock64();
  const unsigned long long w1 = wall_clock64();
  float sum = acc + __uint_as_float(pk);
#pragma unroll
  for (int e = 0; e < 16; e++) sum += c0[e] + c1[e];
#pragma unroll
  for (int e = 0; e < 8; e++) sum += x[e];
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = sum;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = t1 - t0;
    clocks[1] = (long long)(w1 - w0);
  }
}

// Simulated peers: peer q's push of every tile of this rank's segment "arrives".
__global__ void peers_arrive_kernel(unsigned* arrived, int tiles_per_seg, int R, int rank) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < R * tiles_per_seg && i / tiles_per_seg != rank) tile_notify(arrived + i);
}

int launch_peers_arrive(const RsSide& rs, hipStream_t s) {
  int n = rs.R * rs.tiles_per_seg;
  // nothing arrives for the own segment -- in ring order: for the segment whose chain starts at this rank
  const int none = rs.ring ? (rs.rank + 1) % rs.R : rs.rank;
  hipLaunchKernelGGL(peers_arrive_kernel, dim3((n + 255) / 256), dim3(256), 0, s, rs.arrived, rs.tiles_per_seg, rs.R, none);
  TL_HIP(hipGetLastError());
  return TL_OK;
}

__global__ void __launch_bounds__(256) rs_consumer_kernel(const RsSide p) {
  __shared__ int s_item;
  rs_consumer(p, blockIdx.x, gridDim.x, threadIdx.x, 256, &s_item);
}

// ======================================================================================
// Host side
// ======================================================================================
static thread_local char g_err[512] = "";

// Scratch memory of tl_ag_gemm_static, the entry point for callers that cannot allocate: the 256-byte workspace (status
// word, ticket queue, pacing word) followed by the channel flags.  Every device the library runs on holds its own copy
// of this array until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// address kernels and copies are given is the per-device pointer kept in g_static below.
constexpr size_t kStaticWorkspaceBytes = 256;
constexpr size_t kStaticFlagWords = 4096;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes + kStaticFlagWords * sizeof(unsigned)];

constexpr int kMaxDevices = 64;
struct StaticScratch {
  void* ptr;          // device address of `scratch` on this device
  hipEvent_t cleared; // orders the communication stream behind the clearing of the scratch on the compute stream
};
static StaticScratch g_static[kMaxDevices];

__global__ void clear_words_kernel(unsigned* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// Once per device, from tl_ctx_create, with that device current.
static int setup_static_scratch(int dev) {
  if (dev < 0 || dev >= kMaxDevices) return TL_OK;   // such a device simply has no static entry point
  if (g_static[dev].ptr) return TL_OK;
  void* ptr = nullptr;
  TL_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
  hipEvent_t ev;
  TL_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
  g_static[dev].cleared = ev;
  g_static[dev].ptr = ptr;
  return TL_OK;
}

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}


// Segment whose rows GEMM+ReduceScatter computes first: the next rank's in ring order (its own comes last,
// as in a ring reduce-scatter), or its own (so that the reduction of the own segment, the heaviest piece of
// the communication side, overlaps the remaining GEMM tiles and only a push is left at the end).
static int rs_first_rank(const tl_config& c) { return c.tile_order >= TL_ORDER_OWN_FIRST ? c.rank : (c.rank + 1) % c.world_size; }

int resolve_dense(const tl_ctx* ctx, int op, int M, int N, int K, Resolved* r, bool paired_columns) {
  const tl_config& c = ctx->cfg;
  if (M <= 0 || N <= 0 || K <= 0) return fail(TL_ERR_INVALID_ARG, "M, N, K must be positive (got %d, %d, %d)", M, N, K);
  const int R = c.world_size;
  if (M % R) return fail(TL_ERR_UNSUPPORTED_SHAPE, "world size %d must divide M=%d", R, M);
  if (K % 8) return fail(TL_ERR_UNSUPPORTED_SHAPE, "K=%d must be a multiple of 8 (rows of 16-byte pieces)", K);  // a short last K step is zero-filled
  if (N % 8) return fail(TL_ERR_UNSUPPORTED_SHAPE, "N=%d must be a multiple of 8", N);
  if (paired_columns && N % 64) return fail(TL_ERR_UNSUPPORTED_SHAPE, "gate and up columns alternate in blocks of 32: 2F=%d must be a multiple of 64", N);
  memset(r, 0, sizeof *r);
  // ---- compute tile
  int v = -1;
  if (c.tile_m || c.tile_n) {
    for (int i = 0; i < TILE_VARIANTS; i++)
      if (kTileM[i] == c.tile_m && kTileN[i] == c.tile_n) v = i;
    if (v < 0) return fail(TL_ERR_UNSUPPORTED_SHAPE, "compute tile %dx%d is not one of 256x256, 256x224, 128x128", c.tile_m, c.tile_n);
  } else if ((long)M * N <= 1024L * 1024L) {
    v = TILE_128x128;
  } else {
    // 256x256 unless the 224-wide tile divides N and fills the last round of workgroups much better: its wave tile
    // (32x224) reads more LDS bytes per flop and the kernel takes all 256 vector registers, which keeps side-kernel
    // waves off its compute units; measured on 8192x3584x8192, 448 tiles of 256x256 (1.75 rounds) beat 512 of 256x224
    auto fill = [&](int tm, int tn) {
      long tiles = (long)ceil_div(M, tm) * ceil_div(N, tn), G = ctx->num_cus;
      return (double)((long)M * N) / ((double)((tiles + G - 1) / G * G) * tm * tn);
    };
    v = (!paired_columns && N % 224 == 0 && fill(256, 224) > 1.25 * fill(256, 256)) ? TILE_256x224 : TILE_256x256;
  }
  if (paired_columns && v == TILE_256x224) return fail(TL_ERR_UNSUPPORTED_SHAPE, "the gated epilogue pairs 32-wide column blocks: the 256x224 tile has seven per wave");
  r->variant = v;
  r->tile_m = kTileM[v];
  r->tile_n = kTileN[v];
  r->threads = kThreads[v];
  r->lds_bytes = kLds[v];
  r->nbm = ceil_div(M, r->tile_m);
  r->nbn = ceil_div(N, r->tile_n);
  r->n_tiles = r->nbm * r->nbn;
  r->rows_per_rank = M / R;
  // ---- grid
  int G = c.compute_workgroups > 0 ? c.compute_workgroups : ctx->num_cus;
  // The runtime's copy path runs as kernels too, and a persistent GEMM grid that fills every compute unit while it
  // waits for those copies would keep them from ever starting: leave some compute units free for them.
  if (c.compute_workgroups == 0 && c.comm_mode == TL_COMM_STREAM && op == TL_OP_AG_GEMM && G > 32) G -= 16;
  if (G > r->n_tiles) G = r->n_tiles;
  r->G = G;
  {
    // group of row blocks walked together: a power of two that keeps a group inside one rank's rows
    int per_rank = (r->nbm % R == 0) ? r->nbm / R : r->nbm;
    int gm = c.group_m;
    if (gm <= 0) {
      gm = 1;
      while (gm < 4 && per_rank % (gm * 2) == 0) gm *= 2;
    }
    if (gm > r->nbm) gm = r->nbm;
    r->group_m = gm;
  }
  // in-kernel communication workgroups each take a compute unit's worth of LDS and registers; as a kernel of
  // their own they are small and share compute units with the GEMM, so many more of them pay off
  // (the reduce side as a kernel of its own: one workgroup per compute unit, each is bound by the bytes it keeps in flight)
  int n_comm = c.comm_workgroups > 0 ? c.comm_workgroups : (c.comm_mode == TL_COMM_WAVES ? 16 : (op == TL_OP_GEMM_RS ? 256 : 128));
  r->n_comm = (c.comm_mode == TL_COMM_NONE) ? 0 : n_comm;
  // ---- communication tiles
  if (op == TL_OP_AG_GEMM) {
    const int C = c.channels_per_rank;
    // the consumer's wait set is a 64-bit mask over the global channel index
    if ((long)R * C > 64) return fail(TL_ERR_UNSUPPORTED_SHAPE, "world size %d x channels per rank %d = %ld channels; at most 64 are supported", R, C, (long)R * C);
    if (r->rows_per_rank % C) return fail(TL_ERR_UNSUPPORTED_SHAPE, "channels per rank %d must divide M/R=%d", C, r->rows_per_rank);
    r->rows_per_channel = r->rows_per_rank / C;
    int Tm_p = c.comm_tile_m;
    if (Tm_p == 0) {
      Tm_p = r->rows_per_channel;
      // small row tiles: many producer tiles per channel keeps all copy workgroups busy.  With simulated links only the
      // tiles that are due are being copied, a handful at a time and each by one workgroup at the pace of its own memory
      // latency: smaller tiles keep that copy short against the time the link takes for the tile.
      const int floor_rows = c.link_gbps > 0 ? 8 : 32;
      while (Tm_p > floor_rows && Tm_p % 2 == 0) Tm_p /= 2;
      if (r->rows_per_channel % Tm_p) Tm_p = r->rows_per_channel;
    }
    if (Tm_p <= 0 || r->rows_per_channel % Tm_p)
      return fail(TL_ERR_UNSUPPORTED_SHAPE, "producer row tile %d must divide the rows per channel M/(R*C)=%d", Tm_p, r->rows_per_channel);
    int Tn_p = c.comm_tile_n ? c.comm_tile_n : K;
    if (Tn_p <= 0 || K % Tn_p || Tn_p % 8) return fail(TL_ERR_UNSUPPORTED_SHAPE, "producer column tile %d must divide K=%d and be a multiple of 8", Tn_p, K);
    // K chunks: only where the producers are certain to be resident beside the GEMM workgroups (a tile that is already
    // in its K loop waits without helping them), i.e. the 256x256 tile with in-kernel or side-kernel producers
    r->k_chunks = 1;
    if (c.ag_k_chunks >= 2) {
      if (c.comm_tile_n) return fail(TL_ERR_INVALID_ARG, "ag_k_chunks sets the producer column tile itself: comm_tile_n must be 0");
      if (K % (64 * c.ag_k_chunks) || K / (64 * c.ag_k_chunks) < 8)
        return fail(TL_ERR_UNSUPPORTED_SHAPE, "ag_k_chunks=%d needs K=%d to be a multiple of %d with at least 8 steps of 64 per chunk", c.ag_k_chunks, K, 64 * c.ag_k_chunks);
      if (v == TILE_256x256 && (c.comm_mode == TL_COMM_WAVES || c.comm_mode == TL_COMM_SIDE_KERNEL)) {
        r->k_chunks = c.ag_k_chunks;
        Tn_p = K / r->k_chunks;
        if (c.comm_tile_m == 0) {
          // fewer, taller producer tiles: a tile is as many bytes as without chunks
          const int cap = (c.link_gbps > 0 ? 8 : 32) * r->k_chunks;
          while (Tm_p * 2 <= r->rows_per_channel && r->rows_per_channel % (Tm_p * 2) == 0 && Tm_p * 2 <= cap) Tm_p *= 2;
        }
      }
    }
    r->Tm_p = Tm_p;
    r->Tn_p = Tn_p;
    r->n_ptm = M / Tm_p;
    r->n_ptn = K / Tn_p;
    r->expected = r->k_chunks > 1 ? r->rows_per_channel / Tm_p : (r->rows_per_channel / Tm_p) * r->n_ptn;
    r->first_block = 0;
    if (c.tile_order != TL_ORDER_NATURAL) {
      if (r->nbm % R == 0) r->first_block = c.rank * (r->nbm / R);
      // arrival order needs whole row blocks per rank; else it is the ring
      if (c.tile_order == TL_ORDER_ARRIVAL && r->nbm % R == 0 && R > 1) r->arrival_bpr = r->nbm / R;
    }
  } else {
    int Tm_r = c.comm_tile_m;
    if (Tm_r == 0) {   // the GEMM tile's rows, or the largest divisor of M/R below that
      Tm_r = r->tile_m <= r->rows_per_rank ? r->tile_m : r->rows_per_rank;
      while (Tm_r > 1 && r->rows_per_rank % Tm_r) Tm_r--;
    }
    int Tn_r = c.comm_tile_n ? c.comm_tile_n : (N % r->tile_n == 0 ? r->tile_n : N);
    if (Tm_r <= 0 || r->rows_per_rank % Tm_r) return fail(TL_ERR_UNSUPPORTED_SHAPE, "reduce row tile %d must divide M/R=%d", Tm_r, r->rows_per_rank);
    if (Tn_r <= 0 || N % Tn_r || Tn_r % 8) return fail(TL_ERR_UNSUPPORTED_SHAPE, "reduce column tile %d must divide N=%d and be a multiple of 8", Tn_r, N);
    r->Tm_p = Tm_r;
    r->Tn_p = Tn_r;
    r->n_ptm = M / Tm_r;
    r->n_ptn = N / Tn_r;
    r->expected = 0;
    r->first_block = 0;
    if (c.tile_order != TL_ORDER_NATURAL && r->nbm % R == 0) r->first_block = rs_first_rank(c) * (r->nbm / R);
  }
  return TL_OK;
}

static Sched make_sched(const tl_ctx* ctx, const Resolved& r, int op) {
  Sched s;
  s.nbm = r.nbm;
  s.nbn = r.nbn;
  s.n_tiles = r.n_tiles;
  s.G = r.G;
  s.first_block = r.first_block;
  s.swizzle = ctx->cfg.xcd_swizzle;
  s.group_m = r.group_m;
  s.arrival_bpr = r.arrival_bpr;
  s.busy_first = op == TL_OP_AG_GEMM ? 1 : 0;   // the AllGather's consumer: its first tiles wait for rows that arrive in logical order
  return s;
}

static int launch_ag_gemm(int variant, const AgGemmParams& p, int grid, hipStream_t s) {
  if (p.act) {
    if (variant == TILE_256x256) return launch_fused<Cfg256x256>(ag_gemm_kernel<Cfg256x256, true>, p, grid, s);
    if (variant == TILE_128x128) return launch_fused<Cfg128x128>(ag_gemm_kernel<Cfg128x128, true>, p, grid, s);
    return fail(TL_ERR_UNSUPPORTED_SHAPE, "the gated epilogue needs the 256x256 or the 128x128 tile");
  }
  switch (variant) {
    case TILE_256x256: return launch_fused<Cfg256x256>(ag_gemm_kernel<Cfg256x256>, p, grid, s);
    case TILE_256x224: return launch_fused<Cfg256x224>(ag_gemm_kernel<Cfg256x224>, p, grid, s);
    default: return launch_fused<Cfg128x128>(ag_gemm_kernel<Cfg128x128>, p, grid, s);
  }
}

static int launch_gemm_rs(int variant, const GemmRsParams& p, int grid, hipStream_t s) {
  switch (variant) {
    case TILE_256x256: return launch_fused<Cfg256x256>(gemm_rs_kernel<Cfg256x256>, p, grid, s);
    case TILE_256x224: return launch_fused<Cfg256x224>(gemm_rs_kernel<Cfg256x224>, p, grid, s);
    default: return launch_fused<Cfg128x128>(gemm_rs_kernel<Cfg128x128>, p, grid, s);
  }
}

}  // namespace tl

using namespace tl;

extern "C" {

const char* tl_last_error(void) { return g_err; }
const char* tl_version(void) { return "tilelink_mi355 0.2 (gfx950)"; }

static int check_config(const tl_config* cfg) {
  if (cfg->world_size < 1 || cfg->world_size > kMaxWorld) return fail(TL_ERR_INVALID_ARG, "world_size %d outside [1,%d]", cfg->world_size, kMaxWorld);
  if (cfg->rank < 0 || cfg->rank >= cfg->world_size) return fail(TL_ERR_INVALID_ARG, "rank %d outside [0,%d)", cfg->rank, cfg->world_size);
  if (cfg->channels_per_rank < 1) return fail(TL_ERR_INVALID_ARG, "channels_per_rank must be >= 1");
  if (cfg->comm_mode < TL_COMM_NONE || cfg->comm_mode > TL_COMM_COPY_ENGINE) return fail(TL_ERR_INVALID_ARG, "unknown comm_mode %d", cfg->comm_mode);
  if (cfg->tile_order < TL_ORDER_NATURAL || cfg->tile_order > TL_ORDER_ARRIVAL) return fail(TL_ERR_INVALID_ARG, "unknown tile_order %d", cfg->tile_order);
  if (cfg->link_gbps < 0) return fail(TL_ERR_INVALID_ARG, "link_gbps must not be negative");
  if (cfg->comm_workgroups < 0 || cfg->compute_workgroups < 0 || cfg->comm_tile_m < 0 || cfg->comm_tile_n < 0 || cfg->group_m < 0)
    return fail(TL_ERR_INVALID_ARG, "negative workgroup count or tile size");
  return TL_OK;
}

int tl_ctx_create(const tl_config* cfg, tl_ctx** out) {
  if (!cfg || !out) return fail(TL_ERR_INVALID_ARG, "cfg and out must not be null");
  if (int e = check_config(cfg)) return e;
  int dev = 0;
  TL_HIP(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  TL_HIP(hipGetDeviceProperties(&prop, dev));
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return fail(TL_ERR_HIP, "device %d is %s; this library is built for gfx950 only", dev, prop.gcnArchName);
  {
    static std::mutex m;   // contexts may be created from several threads
    std::lock_guard<std::mutex> lock(m);
    if (int e = setup_static_scratch(dev)) return e;
  }
  tl_ctx* c = new tl_ctx;
  c->cfg = *cfg;
  c->device = dev;
  c->num_cus = prop.multiProcessorCount;
  *out = c;
  return TL_OK;
}

int tl_ctx_create_host(const tl_config* cfg, int num_compute_units, tl_ctx** out) {
  if (!cfg || !out) return fail(TL_ERR_INVALID_ARG, "cfg and out must not be null");
  if (num_compute_units < 1) return fail(TL_ERR_INVALID_ARG, "num_compute_units must be positive");
  if (int e = check_config(cfg)) return e;
  tl_ctx* c = new tl_ctx;
  c->cfg = *cfg;
  c->device = -1;   // no device behind it: queries only
  c->num_cus = num_compute_units;
  *out = c;
  return TL_OK;
}

int tl_ctx_destroy(tl_ctx* ctx) {
  delete ctx;
  return TL_OK;
}

int tl_resolve(const tl_ctx* ctx, int op, const long long* dims, int* info) {
  if (int e = check_ctx(ctx)) return e;
  if (!dims || !info) return fail(TL_ERR_INVALID_ARG, "dims and info must not be null");
  if (op != TL_OP_AG_GEMM && op != TL_OP_GEMM_RS) return fail(TL_ERR_INVALID_ARG, "tl_resolve: operator %d has no dense tile geometry", op);
  Resolved r;
  if (int e = resolve_dense(ctx, op, (int)dims[0], (int)dims[1], (int)dims[2], &r)) return e;
  int v[14] = {r.tile_m, r.tile_n, 64, r.G, r.n_comm, r.Tm_p, r.Tn_p, r.n_tiles, r.n_ptm * r.n_ptn, r.expected, r.threads, r.lds_bytes, r.group_m,
               r.k_chunks > 0 ? r.k_chunks : 1};
  memcpy(info, v, sizeof v);
  return TL_OK;
}

int tl_query_workspace(const tl_ctx* ctx, int op, const long long* dims, size_t* ws_bytes, size_t* n_flags) {
  if (int e = check_ctx(ctx)) return e;
  if (!dims || !ws_bytes || !n_flags) return fail(TL_ERR_INVALID_ARG, "dims, ws_bytes and n_flags must not be null");
  if (op == TL_OP_AG_GEMM || op == TL_OP_GEMM_RS) {
    Resolved r;
    if (int e = resolve_dense(ctx, op, (int)dims[0], (int)dims[1], (int)dims[2], &r)) return e;
    *ws_bytes = 256;  // status word (+ padding)
    if (op == TL_OP_AG_GEMM) {
      *n_flags = (size_t)ctx->cfg.world_size * ctx->cfg.channels_per_rank * r.k_chunks;
    } else {
      size_t tiles_per_seg = (size_t)(r.rows_per_rank / r.Tm_p) * r.n_ptn;
      *n_flags = (size_t)r.n_ptm * r.n_ptn + 2 * (size_t)ctx->cfg.world_size * tiles_per_seg;
    }
    return TL_OK;
  }
  if (op == TL_OP_MOE_AG_GATHER_GEMM || op == TL_OP_MOE_GEMM_SCATTER_RS) {
    int info[8];
    if (int e = tl_moe_query(ctx, op, (int)dims[0], (int)dims[1], (int)dims[2], (int)dims[3], (int)dims[4], info)) return e;
    *n_flags = (size_t)info[3];
    *ws_bytes = (size_t)info[4];
    return TL_OK;
  }
  if (op == TL_OP_SP_AG_ATTENTION) {
    int info[8];
    if (int e = tl_attn_query(ctx, (int)dims[0], (int)dims[1], (int)dims[2], 1, info)) return e;
    *n_flags = (size_t)info[2];
    *ws_bytes = (size_t)info[3];
    return TL_OK;
  }
  return fail(TL_ERR_INVALID_ARG, "unknown operator %d", op);
}

int tl_mfma_peak_probe(tl_ctx* ctx, const void* operands, size_t operand_bytes, int iters, float* sink, long long* clocks, void* stream,
                       double* flop) {
  if (int e = check_op_ctx(ctx)) return e;
  if (!operands || !sink || !clocks || iters <= 0) return fail(TL_ERR_INVALID_ARG, "tl_mfma_peak_probe: null pointer or non-positive iteration count");
  const size_t need = (size_t)ctx->num_cus * 512 * 6 * 16;
  if (operand_bytes < need) return fail(TL_ERR_WORKSPACE_TOO_SMALL, "tl_mfma_peak_probe: %zu operand bytes given, %zu needed", operand_bytes, need);
  if (!aligned16(operands)) return fail(TL_ERR_INVALID_ARG, "tl_mfma_peak_probe: operands must be 16-byte aligned");
  hipLaunchKernelGGL(mfma_peak_kernel, dim3(ctx->num_cus), dim3(512), 0, (hipStream_t)stream, (const u32x4*)operands, sink, iters, clocks);
  TL_HIP(hipGetLastError());
  if (flop) *flop = (double)ctx->num_cus * 8.0 * iters * 8.0 * 32768.0;   // workgroups x waves x iterations x MFMAs x (2 x 32 x 32 x 16)
  return TL_OK;
}

int tl_issue_probe(tl_ctx* ctx, int with_mfma, int mode, int iters, float* sink, long long* clocks, void* stream, double* slots) {
  if (int e = check_op_ctx(ctx)) return e;
  if (!sink || !clocks || iters <= 0) return fail(TL_ERR_INVALID_ARG, "tl_issue_probe: null pointer or non-positive iteration count");
  if (mode < 0 || mode > 4) return fail(TL_ERR_INVALID_ARG, "tl_issue_probe: mode %d outside [0,4]", mode);
  const dim3 grid(ctx->num_cus), block(512);
  hipStream_t st = (hipStream_t)stream;
#define TL_PROBE(M, D) hipLaunchKernelGGL((issue_probe_kernel<M, D>), grid, block, 0, st, sink, iters, clocks)
  if (with_mfma) {
    switch (mode) { case 0: TL_PROBE(1, 0); break; case 1: TL_PROBE(1, 1); break; case 2: TL_PROBE(1, 2); break; case 3: TL_PROBE(1, 3); break; default: TL_PROBE(1, 4); }
  } else {
    switch (mode) { case 0: TL_PROBE(0, 0); break; case 1: TL_PROBE(0, 1); break; case 2: TL_PROBE(0, 2); break; case 3: TL_PROBE(0, 3); break; default: TL_PROBE(0, 4); }
  }
#undef TL_PROBE
  TL_HIP(hipGetLastError());
  if (slots) *slots = (double)iters * 8.0;   // slots per wave; every SIMD runs two waves
  return TL_OK;
}

int tl_read_clocks(tl_ctx* ctx, void* workspace, long long* out) {
  if (int e = check_op_ctx(ctx)) return e;
  if (!workspace && ctx->device < kMaxDevices) workspace = g_static[ctx->device].ptr;
  if (!workspace || !out) return fail(TL_ERR_INVALID_ARG, "workspace or out is null");
  TL_HIP(hipMemcpy(out, (const char*)workspace + 32, 2 * sizeof(long long), hipMemcpyDeviceToHost));
  return TL_OK;
}

int tl_check_status(tl_ctx* ctx, void* workspace) {
  if (int e = check_op_ctx(ctx)) return e;
  if (!workspace && ctx->device < kMaxDevices) workspace = g_static[ctx->device].ptr;   // the scratch of tl_ag_gemm_static
  if (!workspace) return fail(TL_ERR_INVALID_ARG, "workspace is null");
  int st = 0;
  TL_HIP(hipMemcpy(&st, workspace, sizeof st, hipMemcpyDeviceToHost));
  if (st != 0) {
    int zero = 0;
    TL_HIP(hipMemcpy(workspace, &zero, sizeof zero, hipMemcpyHostToDevice));
    return fail(TL_ERR_TIMEOUT, "a flag wait expired (flag index %d)", st - 1);
  }
  return TL_OK;
}

static int ag_gemm_impl(tl_ctx* ctx, const void* const* a_shards, void* a_gathered, const void* b, void* c, int M, int N, int K, int act,
                        unsigned* flags, unsigned epoch, void* workspace, size_t ws_bytes, void* compute_stream, void* comm_stream,
                        void* const* peer_slots = nullptr) {
  if (int e = check_op_ctx(ctx)) return e;
  const tl_config& cfg = ctx->cfg;
  if (!a_shards || !a_gathered || !b || !c || !flags || !workspace) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm: null pointer argument");
  if (epoch == 0) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm: epoch starts at 1");
  Resolved r;
  if (int e = resolve_dense(ctx, TL_OP_AG_GEMM, M, N, K, &r, act != 0)) return e;
  if (ws_bytes < 256) return fail(TL_ERR_WORKSPACE_TOO_SMALL, "tl_ag_gemm: workspace of %zu bytes, 256 needed", ws_bytes);
  const int R = cfg.world_size;
  if (!aligned16(a_gathered) || !aligned16(b) || !aligned16(c)) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm: device pointers must be 16-byte aligned");
  for (int q = 0; q < R; q++)
    if (!a_shards[q] || !aligned16(a_shards[q])) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm: a_shards[%d] is null or misaligned", q);

  AgGemmParams p;
  memset(&p, 0, sizeof p);
  fill_ag_producer(ctx, &p.prod, a_shards, a_gathered, K, r.Tm_p, r.Tn_p, r.n_ptm, r.n_ptn, r.rows_per_rank, r.rows_per_channel,
                   flags, epoch, workspace);
  // the queue hands out the shards in the order in which the GEMM reads them: the owner of the schedule's first row
  // block first (the local shard under the rotated orders: nothing to copy if it is in place, so its channels are
  // ready at once), then along the ring
  p.prod.first_src = r.first_block / (r.nbm / R > 0 ? r.nbm / R : 1) % R;
  p.prod.k_chunks = r.k_chunks;
  if (r.arrival_bpr) p.prod.interleave = 1;  // the queue follows the order in which the GEMM reads
  if (peer_slots) {
    // push mode: behind the tiles that arrive here, one ticket per (producer tile of the local shard, peer)
    if (cfg.comm_mode != TL_COMM_WAVES && cfg.comm_mode != TL_COMM_SIDE_KERNEL)
      return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm_push: comm_mode must be TL_COMM_WAVES or TL_COMM_SIDE_KERNEL");
    if (r.k_chunks > 1 || cfg.link_gbps > 0) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm_push: ag_k_chunks and link_gbps do not apply to the push form");
    for (int q = 0; q < R; q++) {
      if (q != cfg.rank && (!peer_slots[q] || !aligned16(peer_slots[q]))) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm_push: peer_slots[%d] is null or misaligned", q);
      p.prod.peer_slots[q] = (bf16_t*)peer_slots[q];
    }
    p.prod.n_out = (r.rows_per_rank / r.Tm_p) * r.n_ptn * (R - 1);
    p.prod.pushed = flags + (size_t)R * cfg.channels_per_rank * r.k_chunks;
    p.prod.ticket_end = epoch * (unsigned)(r.n_ptm * r.n_ptn + p.prod.n_out);
  }
  p.b = (const bf16_t*)b;
  p.c = (bf16_t*)c;
  p.M = M; p.N = N; p.K = K;
  p.act = act;
  p.sched = make_sched(ctx, r, TL_OP_AG_GEMM);
  hipStream_t cs = (hipStream_t)compute_stream, ms = (hipStream_t)comm_stream;

  const bool alone = cfg.comm_alone != 0;  // communication side only (timing)
  if (r.k_chunks > 1 && cfg.comm_mode != TL_COMM_WAVES && cfg.comm_mode != TL_COMM_SIDE_KERNEL) r.k_chunks = 1;
  if (alone && (cfg.comm_mode == TL_COMM_NONE || cfg.comm_mode == TL_COMM_EXTERNAL))
    return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm: comm_alone needs a comm_mode in which the library runs a producer");
  p.do_compute = alone ? 0 : 1;
  switch (cfg.comm_mode) {
    case TL_COMM_NONE:
      p.n_comm = 0; p.do_wait = 0;
      return launch_ag_gemm(r.variant, p, r.G, cs);
    case TL_COMM_WAVES:
      p.n_comm = r.n_comm; p.do_wait = 1;
      p.prod.wait_target = epoch * (unsigned)r.expected;
      return launch_ag_gemm(r.variant, p, alone ? r.n_comm : r.G + r.n_comm, cs);
    case TL_COMM_EXTERNAL:
      p.n_comm = 0; p.do_wait = 2;
      p.prod.wait_target = epoch * (unsigned)r.expected;
      return launch_ag_gemm(r.variant, p, r.G, cs);
    case TL_COMM_SIDE_KERNEL: {
      // The producer is enqueued first: it waits for nothing, so even if both streams end up on one
      // hardware queue the worst case is that the two kernels run one after the other.
      p.n_comm = 0; p.do_wait = 1;
      p.prod.wait_target = epoch * (unsigned)r.expected;
      hipLaunchKernelGGL(ag_producer_kernel, dim3(r.n_comm), dim3(256), 0, ms, p.prod);
      TL_HIP(hipGetLastError());
      return alone ? TL_OK : launch_ag_gemm(r.variant, p, r.G, cs);
    }
    case TL_COMM_STREAM:
    case TL_COMM_COPY_ENGINE: {
      // rank_copy_data + rank_notify per source rank, ring order: through the runtime's copy kernels, or through a copy
      // engine, which takes no compute unit (the copy kind that asks the runtime to keep the compute units out of it)
      p.n_comm = 0; p.do_wait = 2;
      p.prod.wait_target = epoch;
      const hipMemcpyKind kind = cfg.comm_mode == TL_COMM_COPY_ENGINE ? hipMemcpyDeviceToDeviceNoCU : hipMemcpyDeviceToDevice;
      const size_t shard_bytes = (size_t)r.rows_per_rank * K * sizeof(bf16_t);
      for (int i = 0; i < R; i++) {
        int q = (cfg.rank + i) % R;  // local shard first (it is usually free), then rank+1, ...
        char* dst = (char*)a_gathered + (size_t)q * shard_bytes;
        if (!(q == cfg.rank && p.prod.local_in_place)) TL_HIP(hipMemcpyAsync(dst, a_shards[q], shard_bytes, kind, ms));
        hipLaunchKernelGGL(notify_kernel, dim3((cfg.channels_per_rank + 63) / 64), dim3(64), 0, ms, flags + q * cfg.channels_per_rank, cfg.channels_per_rank, 1u);
        TL_HIP(hipGetLastError());
      }
      return alone ? TL_OK : launch_ag_gemm(r.variant, p, r.G, cs);
    }
  }
  return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm: unknown comm_mode");
}

int tl_ag_gemm(tl_ctx* ctx, const void* const* a_shards, void* a_gathered, const void* b, void* c, int M, int N, int K,
               unsigned* flags, unsigned epoch, void* workspace, size_t ws_bytes, void* compute_stream, void* comm_stream) {
  return ag_gemm_impl(ctx, a_shards, a_gathered, b, c, M, N, K, 0, flags, epoch, workspace, ws_bytes, compute_stream, comm_stream);
}

int tl_ag_gemm_static(tl_ctx* ctx, const void* const* a_shards, void* a_gathered, const void* b, void* c, int M, int N, int K,
                      void* compute_stream, void* comm_stream) {
  if (int e = check_op_ctx(ctx)) return e;
  int cur = -1;
  TL_HIP(hipGetDevice(&cur));
  if (cur != ctx->device) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm_static: the context belongs to device %d, the current device is %d", ctx->device, cur);
  if (cur >= kMaxDevices || !g_static[cur].ptr) return fail(TL_ERR_HIP, "tl_ag_gemm_static: no static scratch was set up for device %d", cur);
  Resolved r;
  if (int e = resolve_dense(ctx, TL_OP_AG_GEMM, M, N, K, &r)) return e;
  const size_t n_flags = (size_t)ctx->cfg.world_size * ctx->cfg.channels_per_rank * (r.k_chunks > 0 ? r.k_chunks : 1);
  if (n_flags > kStaticFlagWords)
    return fail(TL_ERR_WORKSPACE_TOO_SMALL, "tl_ag_gemm_static: %zu channel flags needed, the static scratch holds %zu; use tl_ag_gemm with a caller's workspace", n_flags, kStaticFlagWords);
  unsigned* ws = (unsigned*)g_static[cur].ptr;
  unsigned* flags = ws + kStaticWorkspaceBytes / sizeof(unsigned);
  hipStream_t cs = (hipStream_t)compute_stream, ms = (hipStream_t)comm_stream;
  // The scratch keeps the last call's counters: start from zero (a fill kernel, which a captured graph replays
  // faithfully), and let the communication stream's producers start behind it.
  const int n_clear = (int)(kStaticWorkspaceBytes / sizeof(unsigned) + n_flags);
  hipLaunchKernelGGL(clear_words_kernel, dim3((n_clear + 255) / 256), dim3(256), 0, cs, ws, n_clear);
  TL_HIP(hipGetLastError());
  if (ms != cs) {
    TL_HIP(hipEventRecord(g_static[cur].cleared, cs));
    TL_HIP(hipStreamWaitEvent(ms, g_static[cur].cleared, 0));
  }
  return ag_gemm_impl(ctx, a_shards, a_gathered, b, c, M, N, K, 0, flags, 1u, ws, kStaticWorkspaceBytes, compute_stream, comm_stream);
}

int tl_ag_gemm_act_mul(tl_ctx* ctx, const void* const* a_shards, void* a_gathered, const void* b_gate_up, void* y, int M, int F, int K, int act,
                       unsigned* flags, unsigned epoch, void* workspace, size_t ws_bytes, void* compute_stream, void* comm_stream) {
  if (act != TL_ACT_SILU_MUL && act != TL_ACT_GELU_MUL) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm_act_mul: unknown activation %d", act);
  if (F <= 0 || F > (1 << 29)) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm_act_mul: F=%d out of range", F);
  static_assert(TL_ACT_SILU_MUL == ACT_SILU_MUL && TL_ACT_GELU_MUL == ACT_GELU_MUL, "activation codes");
  return ag_gemm_impl(ctx, a_shards, a_gathered, b_gate_up, y, M, 2 * F, K, act, flags, epoch, workspace, ws_bytes, compute_stream, comm_stream);
}

int tl_ag_gemm_push(tl_ctx* ctx, const void* const* a_shards, void* a_gathered, void* const* peer_slots, const void* b, void* c, int M, int N,
                    int K, unsigned* flags, unsigned epoch, void* workspace, size_t ws_bytes, void* compute_stream, void* comm_stream) {
  if (!peer_slots) return fail(TL_ERR_INVALID_ARG, "tl_ag_gemm_push: peer_slots is null");
  return ag_gemm_impl(ctx, a_shards, a_gathered, b, c, M, N, K, 0, flags, epoch, workspace, ws_bytes, compute_stream, comm_stream, peer_slots);
}

}  // extern "C"

// tl_gemm_rs and its ring variant.  `ring`: peer_recv[q] is the running sum of segment q handed on by the next rank (none
// for segment rank+1, whose chain starts here), peer_push[q] the landing zone of the previous rank (none for the own
// segment, whose sum ends in `out`); the GEMM and the reduce side walk the segments in chain order rank+1, rank+2, ..., rank.
static int gemm_rs_impl(const char* name, bool ring, tl_ctx* ctx, const void* a, const void* b, void* partial, const void* const* peer_recv,
                        void* const* peer_push, void* out, int M, int N, int K, unsigned* flags, unsigned epoch, void* workspace,
                        size_t ws_bytes, void* compute_stream, void* comm_stream) {
  if (int e = check_op_ctx(ctx)) return e;
  const tl_config& cfg = ctx->cfg;
  if (!a || !b || !partial || !peer_recv || !peer_push || !out || !flags || !workspace) return fail(TL_ERR_INVALID_ARG, "%s: null pointer argument", name);
  if (epoch == 0) return fail(TL_ERR_INVALID_ARG, "%s: epoch starts at 1", name);
  Resolved r;
  if (int e = resolve_dense(ctx, TL_OP_GEMM_RS, M, N, K, &r)) return e;
  if (ws_bytes < 256) return fail(TL_ERR_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes, 256 needed", name, ws_bytes);
  const int R = cfg.world_size;
  if (!aligned16(a) || !aligned16(b) || !aligned16(partial) || !aligned16(out)) return fail(TL_ERR_INVALID_ARG, "%s: device pointers must be 16-byte aligned", name);
  const int no_recv = ring ? (cfg.rank + 1) % R : cfg.rank;   // the segment nothing is received for
  for (int q = 0; q < R; q++) {
    if (q != no_recv && (!peer_recv[q] || !aligned16(peer_recv[q]))) return fail(TL_ERR_INVALID_ARG, "%s: peer_recv[%d] is null or misaligned", name, q);
    if (q != cfg.rank && (!peer_push[q] || !aligned16(peer_push[q]))) return fail(TL_ERR_INVALID_ARG, "%s: peer_push[%d] is null or misaligned", name, q);
  }

  GemmRsParams p;
  memset(&p, 0, sizeof p);
  p.a = (const bf16_t*)a; p.b = (const bf16_t*)b; p.K = K;
  int first_rank = rs_first_rank(cfg);
  if (ring) {
    first_rank = no_recv;
    if (cfg.tile_order != TL_ORDER_NATURAL && r.nbm % R == 0) r.first_block = first_rank * (r.nbm / R);
  }
  p.sched = make_sched(ctx, r, TL_OP_GEMM_RS);
  fill_rs_side(ctx, &p.rs, partial, peer_recv, peer_push, out, M, N, r.tile_m, r.tile_n, r.Tm_p, r.Tn_p, flags, epoch, workspace);
  if (cfg.tile_order != TL_ORDER_NATURAL) p.rs.rs_first_block = first_rank * (r.rows_per_rank / r.Tm_p);
  if (ring) {
    p.rs.ring = 1;
    p.rs.direct = 0;   // every segment passes through the reduce side
    if (R > 1 && !aligned128(peer_recv[cfg.rank])) p.rs.ctl.strict = 1;
  }
  hipStream_t cs = (hipStream_t)compute_stream, ms = (hipStream_t)comm_stream;
  auto peers_arrive = [&](hipStream_t s) -> int { return launch_peers_arrive(p.rs, s); };

  const bool alone = cfg.comm_alone != 0;  // reduce/push side only, on a partial product that is already complete
  p.do_compute = alone ? 0 : 1;
  switch (cfg.comm_mode) {
    case TL_COMM_NONE:
      if (alone) return fail(TL_ERR_INVALID_ARG, "%s: comm_alone needs a comm_mode with a reduce side", name);
      p.n_comm = 0; p.do_notify = 0; p.rs.do_wait = 0;
      if (p.rs.direct == 2) p.rs.direct = 1;  // no reduce side at all in this mode
      return launch_gemm_rs(r.variant, p, r.G, cs);
    case TL_COMM_WAVES:
      if (int e = peers_arrive(alone ? cs : ms)) return e;
      p.n_comm = r.n_comm; p.do_notify = alone ? 0 : 1; p.rs.do_wait = alone ? 0 : 1;
      return launch_gemm_rs(r.variant, p, alone ? r.n_comm : r.G + r.n_comm, cs);
    case TL_COMM_EXTERNAL:
      return fail(TL_ERR_INVALID_ARG, "%s: TL_COMM_EXTERNAL is not defined for this operator", name);
    case TL_COMM_COPY_ENGINE:
      return fail(TL_ERR_INVALID_ARG, "%s: TL_COMM_COPY_ENGINE is an AllGather binding; the reduction needs compute units", name);
    case TL_COMM_STREAM:
    case TL_COMM_SIDE_KERNEL: {
      // The GEMM kernel is enqueued before the reduce kernel that waits on it: should both streams share a
      // hardware queue, the reduce kernel then simply runs after the GEMM instead of blocking it.
      p.n_comm = 0; p.do_notify = alone ? 0 : 1; p.rs.do_wait = alone ? 0 : 1;
      // ... and with the own segment reduced in the GEMM's epilogue the GEMM itself waits for the peers' arrival
      if (p.rs.direct == 2)
        if (int e = peers_arrive(ms)) return e;
      if (!alone)
        if (int e = launch_gemm_rs(r.variant, p, r.G, cs)) return e;
      if (p.rs.direct != 2)
        if (int e = peers_arrive(ms)) return e;
      use_rs_queue(&p.rs, workspace, epoch);   // (the GEMM kernel above was given its parameters by value before this)
      hipLaunchKernelGGL(rs_consumer_kernel, dim3(r.n_comm), dim3(256), 0, ms, p.rs);
      TL_HIP(hipGetLastError());
      return TL_OK;
    }
  }
  return fail(TL_ERR_INVALID_ARG, "%s: unknown comm_mode", name);
}

extern "C" {

int tl_gemm_rs(tl_ctx* ctx, const void* a, const void* b, void* partial, const void* const* peer_recv, void* const* peer_push,
               void* out, int M, int N, int K, unsigned* flags, unsigned epoch, void* workspace, size_t ws_bytes,
               void* compute_stream, void* comm_stream) {
  return gemm_rs_impl("tl_gemm_rs", false, ctx, a, b, partial, peer_recv, peer_push, out, M, N, K, flags, epoch, workspace, ws_bytes,
                      compute_stream, comm_stream);
}

int tl_gemm_ring_rs(tl_ctx* ctx, const void* a, const void* b, void* partial, const void* const* ring_recv, void* const* ring_push,
                    void* out, int M, int N, int K, unsigned* flags, unsigned epoch, void* workspace, size_t ws_bytes,
                    void* compute_stream, void* comm_stream) {
  return gemm_rs_impl("tl_gemm_ring_rs", true, ctx, a, b, partial, ring_recv, ring_push, out, M, N, K, flags, epoch, workspace, ws_bytes,
                      compute_stream, comm_stream);
}

int tl_dump_schedule(const tl_ctx* ctx, int op, const long long* dims, int* out, size_t cap, size_t* n) {
  if (int e = check_ctx(ctx)) return e;
  if (!dims || !n) return fail(TL_ERR_INVALID_ARG, "dims and n must not be null");
  if (op != TL_OP_AG_GEMM && op != TL_OP_GEMM_RS) return fail(TL_ERR_INVALID_ARG, "tl_dump_schedule: operator %d has no static schedule", op);
  const int M = (int)dims[0], N = (int)dims[1], K = (int)dims[2];
  Resolved r;
  if (int e = resolve_dense(ctx, op, M, N, K, &r)) return e;
  const tl_config& cfg = ctx->cfg;
  Sched s = make_sched(ctx, r, op);
  size_t need = (op == TL_OP_AG_GEMM) ? (size_t)r.n_tiles * 8 : (size_t)r.n_tiles * 9 + (size_t)r.n_ptm * r.n_ptn * 9;
  *n = need;
  if (!out || cap < need) return fail(TL_ERR_WORKSPACE_TOO_SMALL, "tl_dump_schedule: %zu ints needed, capacity %zu", need, cap);
  int* o = out;
  for (int pos = 0; pos < r.n_tiles; pos++) {
    int t = sched_tile(s, pos);
    int bm = t / r.nbn, bn = t % r.nbn;
    int row_lo = bm * r.tile_m, row_hi = row_lo + r.tile_m < M ? row_lo + r.tile_m : M;
    int col_lo = bn * r.tile_n, col_hi = col_lo + r.tile_n < N ? col_lo + r.tile_n : N;
    if (op == TL_OP_AG_GEMM) {
      int rec[8] = {t, bm, bn, row_lo, row_hi, row_lo / r.rows_per_channel, (row_hi - 1) / r.rows_per_channel, 0};
      memcpy(o, rec, sizeof rec);
      o += 8;
    } else {
      int rec[9] = {t, bm, bn, row_lo, row_hi, row_lo / r.Tm_p, (row_hi - 1) / r.Tm_p, col_lo / r.Tn_p, (col_hi - 1) / r.Tn_p};
      memcpy(o, rec, sizeof rec);
      o += 9;
    }
  }
  if (op == TL_OP_GEMM_RS) {
    int first = cfg.tile_order != TL_ORDER_NATURAL ? rs_first_rank(cfg) * (r.rows_per_rank / r.Tm_p) : 0;
    for (int i = 0; i < r.n_ptm * r.n_ptn; i++) {
      int cm = (i / r.n_ptn + first) % r.n_ptm, cn = i % r.n_ptn;
      int row_lo = cm * r.Tm_p, row_hi = row_lo + r.Tm_p, col_lo = cn * r.Tn_p, col_hi = col_lo + r.Tn_p;
      int n_m = (row_hi - 1) / r.tile_m - row_lo / r.tile_m + 1, n_n = (col_hi - 1) / r.tile_n - col_lo / r.tile_n + 1;
      int rec[9] = {cm * r.n_ptn + cn, cm, cn, row_lo, row_hi, col_lo, col_hi, row_lo / r.rows_per_rank, n_m * n_n};
      memcpy(o, rec, sizeof rec);
      o += 9;
    }
  }
  return TL_OK;
}

}  // extern "C"
