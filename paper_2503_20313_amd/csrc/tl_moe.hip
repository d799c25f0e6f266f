// MoE halves of the tensor-parallel FFN: routing -> dynamic mapping tables, AllGather + gather +
// grouped GEMM, grouped GEMM + scatter + top-k reduce + ReduceScatter.  gfx950 only.
//
// Dynamic mapping (paper, "Tile-Centric Mapping": lookup tables f_S_low, f_S_high, f_R, f_C filled at run
// time by the routing): one table row of 8 ints per grouped-GEMM row tile,
//   (f_S_low, f_S_high, expert, chan_mask_lo, chan_mask_hi, f_R_lo, f_R_hi, 0),
// over the routed rows sorted by expert (stable: ascending row id = token*topk + slot inside an expert).
#include "tl_ag_producer.h"
#include "tl_gemm_tile.h"
#include "tl_host.h"
#include "tl_rs_consumer.h"

namespace tl {

constexpr int kMaxExperts = 64;
constexpr int kMaxTopk = 8;
constexpr int kRouteThreads = 1024;

// ======================================================================================
// Routing, step 1: per token, the k largest gate logits (ties -> lower expert index, listed by
// descending logit) and their softmax weights (over all E experts, renormalised over the k
// selected if asked).  One thread per token.
// ======================================================================================
__global__ void moe_topk_kernel(const float* __restrict__ logits, int T, int E, int topk, int renormalize, int* __restrict__ topk_ids,
                                float* __restrict__ topk_w) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float* row = logits + (long)t * E;
  float mx = row[0];
  for (int e = 1; e < E; e++) mx = fmaxf(mx, row[e]);
  float denom = 0.f;
  for (int e = 0; e < E; e++) denom += expf(row[e] - mx);
  unsigned long long taken = 0;
  float w[kMaxTopk];
  float wsum = 0.f;
  for (int j = 0; j < topk; j++) {
    int best = -1;
    float bv = 0.f;
    for (int e = 0; e < E; e++) {
      if ((taken >> e) & 1) continue;
      float v = row[e];
      if (best < 0 || v > bv) { best = e; bv = v; }  // strict >: the lower index wins a tie
    }
    taken |= 1ull << best;
    topk_ids[(long)t * topk + j] = best;
    w[j] = expf(bv - mx) / denom;
    wsum += w[j];
  }
  for (int j = 0; j < topk; j++) topk_w[(long)t * topk + j] = renormalize ? w[j] / wsum : w[j];
}

// ======================================================================================
// Routing, step 2 (one workgroup of 16 waves): stable counting sort of the routed rows by expert, expert
// offsets, and the tile tables.  Wave w owns a contiguous range of rows and walks it 64 rows at a time; inside
// a step the lanes that route to the same expert are found with one ballot per bit of the expert index, which
// gives every row its rank among them.  Pass A counts rows per (wave, expert); a scan turns the counts into the
// position where each wave's rows of each expert start; pass B places the rows (stable: waves, steps and lanes
// are in row order) and ORs each row's AllGather channel into its tile's mask.
// ======================================================================================
constexpr int kRouteWaves = kRouteThreads / 64;
constexpr int kLdsTiles = 2048;  // tile tables are assembled in LDS up to this many tiles, else in global memory

__device__ __forceinline__ unsigned long long same_expert_lanes(int e, bool valid) {
  unsigned long long same = __builtin_amdgcn_ballot_w64(valid);
#pragma unroll
  for (int b = 0; b < 6; b++) {  // kMaxExperts = 64
    unsigned long long bal = __builtin_amdgcn_ballot_w64(valid && ((e >> b) & 1));
    same &= ((e >> b) & 1) ? bal : ~bal;
  }
  return same;
}

__global__ void __launch_bounds__(kRouteThreads) moe_sort_kernel(const int* __restrict__ topk_ids, int n_rows, int E, int topk, int T, int R, int C,
                                                                 int Tm, int* __restrict__ expert_offsets, int* __restrict__ sorted_row,
                                                                 int* __restrict__ tile_tables, int* __restrict__ n_tiles) {
  __shared__ int s_cnt[kRouteWaves][kMaxExperts];
  __shared__ int s_off[kMaxExperts + 1], s_tbase[kMaxExperts + 1];
  __shared__ unsigned s_mlo[kLdsTiles], s_mhi[kLdsTiles];
  __shared__ int s_rmin[kLdsTiles], s_rmax[kLdsTiles];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = ((n_rows + kRouteWaves - 1) / kRouteWaves + 63) / 64 * 64;
  const int lo = min(wave * chunk, n_rows), hi = min(lo + chunk, n_rows);
  const unsigned long long below = (1ull << lane) - 1;
  for (int i = tid; i < kRouteWaves * kMaxExperts; i += kRouteThreads) (&s_cnt[0][0])[i] = 0;
  __syncthreads();
  // ---- pass A: rows per (wave, expert)
  for (int base = lo; base < hi; base += 64) {
    const int r = base + lane;
    const bool valid = r < hi;
    const int e = valid ? topk_ids[r] : 0;
    const unsigned long long same = same_expert_lanes(e, valid);
    if (valid && (same & below) == 0) s_cnt[wave][e] += __builtin_popcountll(same);  // the group's first lane
  }
  __syncthreads();
  // ---- offsets, tile bases, start position of every (wave, expert)
  if (tid < E) {
    int tot = 0;
    for (int w = 0; w < kRouteWaves; w++) tot += s_cnt[w][tid];
    s_off[tid + 1] = tot;
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0, tb = 0;
    for (int e = 0; e < E; e++) {
      int c = s_off[e + 1];
      s_off[e] = run;
      s_tbase[e] = tb;
      run += c;
      tb += (c + Tm - 1) / Tm;
    }
    s_off[E] = run;
    s_tbase[E] = tb;
    *n_tiles = tb;
  }
  __syncthreads();
  if (tid < E) {
    int run = s_off[tid];
    for (int w = 0; w < kRouteWaves; w++) {
      int c = s_cnt[w][tid];
      s_cnt[w][tid] = run;
      run += c;
    }
  }
  const int nt = s_tbase[E];
  const bool in_lds = nt <= kLdsTiles;
  // ---- tile records: range and expert now, masks and rank span start empty
  for (int tau = tid; tau < nt; tau += kRouteThreads) {
    int e = 0;
    while (s_tbase[e + 1] <= tau) e++;
    int f_lo = s_off[e] + (tau - s_tbase[e]) * Tm;
    int* rec = tile_tables + (long)tau * 8;
    rec[0] = f_lo; rec[1] = min(f_lo + Tm, s_off[e + 1]); rec[2] = e; rec[7] = 0;
    if (in_lds) { s_mlo[tau] = 0; s_mhi[tau] = 0; s_rmin[tau] = R; s_rmax[tau] = -1; }
    else { rec[3] = 0; rec[4] = 0; rec[5] = R; rec[6] = -1; }
  }
  __threadfence();
  __syncthreads();
  // ---- pass B: place the rows, collect each tile's channels and source ranks
  const int tokens_per_rank = T / R, tokens_per_channel = tokens_per_rank / C;
  for (int base = lo; base < hi; base += 64) {
    const int r = base + lane;
    const bool valid = r < hi;
    const int e = valid ? topk_ids[r] : 0;
    const unsigned long long same = same_expert_lanes(e, valid);
    int start = 0;
    if (valid) start = s_cnt[wave][e];
    if (valid && (same & below) == 0) s_cnt[wave][e] = start + __builtin_popcountll(same);
    if (valid) {
      const int pos = start + __builtin_popcountll(same & below);
      sorted_row[pos] = r;
      const int tau = s_tbase[e] + (pos - s_off[e]) / Tm;
      const int token = r / topk, ch = token / tokens_per_channel, q = token / tokens_per_rank;
      if (in_lds) {
        if (ch < 32) atomicOr(&s_mlo[tau], 1u << ch); else atomicOr(&s_mhi[tau], 1u << (ch - 32));
        atomicMin(&s_rmin[tau], q);
        atomicMax(&s_rmax[tau], q);
      } else {
        int* rec = tile_tables + (long)tau * 8;
        if (ch < 32) atomicOr((unsigned*)rec + 3, 1u << ch); else atomicOr((unsigned*)rec + 4, 1u << (ch - 32));
        atomicMin(rec + 5, q);
        atomicMax(rec + 6, q);
      }
    }
  }
  __syncthreads();
  for (int e = tid; e <= E; e += kRouteThreads) expert_offsets[e] = s_off[e];
  if (in_lds)
    for (int tau = tid; tau < nt; tau += kRouteThreads) {
      int* rec = tile_tables + (long)tau * 8;
      rec[3] = (int)s_mlo[tau]; rec[4] = (int)s_mhi[tau]; rec[5] = s_rmin[tau]; rec[6] = s_rmax[tau];
    }
}

// ======================================================================================
// Part 1: AllGather + gather + grouped GEMM.  Output tile = (row tile tau of the sorted rows) x
// (column block of I); its A rows are token rows picked through sorted_row, its B is the expert's W1.
// ======================================================================================
struct MoeP1Params {
  AgProducer prod;          // token shards -> gathered tokens [T,H]
  const bf16_t* w1;         // [E,H,I]
  bf16_t* y1;               // [T*topk, I] in sorted row order
  const int* sorted_row;
  const int* tile_tables;
  const int* n_row_tiles;   // device: number of row tiles (from the routing)
  int H, I, topk;           // I = columns of the GEMM (twice the output features with an activation)
  int act;                  // 0, or ACT_*: W1 holds gate and up columns, y1 = act(gate) * up has I/2 columns
  int nbn, G, group_m, swizzle;
  int n_comm, do_compute, do_wait;
};

// Order of the row tiles of a grouped GEMM: an expert's last row tile is often nearly empty and then, in the 64-row tile
// shape, takes half the time of a full one (it still streams its whole block of the expert's weights) -- so the long
// tiles (more than half the rows valid) go first, in the usual schedule, and the short ones are dealt out afterwards:
// first, two each, to the workgroups that the long tiles leave without work in their last round, then to all in turn.
// perm[0 .. n_long) = the long row tiles in table order, perm[n_long .. n) = the short ones.  Computed by wave 0 of
// every workgroup from the routing tables (a few hundred entries); callers fall back to table order above kMaxPerm.
constexpr int kMaxPerm = 2048;
__device__ __forceinline__ int long_tiles_first(const int* tile_tables, int n, int tile_m, unsigned short* perm, int tid) {
  const int lane = tid & 63;
  int n_long = 0;
  if (__builtin_amdgcn_readfirstlane(tid >> 6) == 0) {
    for (int c = 0; c < n; c += 64) {
      const int i = c + lane;
      const bool is_long = i < n && 2 * (tile_tables[(long)i * 8 + 1] - tile_tables[(long)i * 8]) > tile_m;
      n_long += __builtin_popcountll(__builtin_amdgcn_ballot_w64(is_long));
    }
    int c_long = 0, c_short = 0;
    for (int c = 0; c < n; c += 64) {
      const int i = c + lane;
      const bool valid = i < n;
      const bool is_long = valid && 2 * (tile_tables[(long)i * 8 + 1] - tile_tables[(long)i * 8]) > tile_m;
      const unsigned long long ml = __builtin_amdgcn_ballot_w64(is_long), mv = __builtin_amdgcn_ballot_w64(valid);
      const unsigned long long below = (1ull << lane) - 1;
      if (valid) {
        const int pos = is_long ? c_long + __builtin_popcountll(ml & below) : n_long + c_short + __builtin_popcountll(mv & ~ml & below);
        perm[pos] = (unsigned short)i;
      }
      c_long += __builtin_popcountll(ml);
      c_short += __builtin_popcountll(mv & ~ml);
    }
  }
  return n_long;  // meaningful in wave 0 only: the caller broadcasts it
}

// A row tile of at most 64 rows in the small tile shape with the deeper ring.  Out of line: inlined beside the 256x256
// loop it takes the kernel to 256 registers, which leaves no room for a producer wave beside two of its waves.
template <class Out>
__device__ __attribute__((noinline)) void moe_small_gather_tile(const bf16_t* a, long lda, const int* a_rows, int a_div, const bf16_t* b, long ldb,
                                                                Out out, int rows, int cols, int K, char* smem) {
  gemm_tile<Cfg64x256, Out>(a, lda, a_rows, a_div, b, ldb, out, rows, cols, K, smem);
}

template <class Cfg, bool GATED = false>
__global__ void __launch_bounds__(Cfg::NTHREADS) moe_ag_gather_gemm_kernel(const MoeP1Params p) {
  typedef typename std::conditional<GATED, GatedRows, DenseRows>::type Out;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int s_ticket;
  __shared__ int s_n_long;
  __shared__ unsigned short s_perm[kMaxPerm];
  const int tid = threadIdx.x;
  if ((int)blockIdx.x < p.n_comm) {
    ag_producer(p.prod, tid, Cfg::NTHREADS, &s_ticket);
    return;
  }
  if (!p.do_compute) return;
  __builtin_amdgcn_s_setprio(TL_COMPUTE_WAVE_PRIO);  // matrix waves go first when they share a SIMD with communication waves
  const int w = blockIdx.x - p.n_comm;
  const int n_rt = *p.n_row_tiles;
  constexpr bool kSmallShape = Cfg::BM == 256 && Cfg::BN == 256;   // short tiles are cheaper only where they have a shape of their own
  const bool reorder = kSmallShape && n_rt <= kMaxPerm;
  int n_long = n_rt;
  if (reorder) {
    int nl = long_tiles_first(p.tile_tables, n_rt, Cfg::BM, s_perm, tid);
    if (tid == 0) s_n_long = nl;
    __syncthreads();
    n_long = s_n_long;
  }
  Sched sc;
  sc.nbm = n_long;
  sc.nbn = p.nbn;
  sc.n_tiles = sc.nbm * sc.nbn;
  sc.G = p.G;
  sc.first_block = 0;
  sc.swizzle = p.swizzle;
  sc.group_m = p.group_m < n_long ? p.group_m : (n_long > 0 ? n_long : 1);
  sc.arrival_bpr = 0;
  auto do_tile = [&](int bm, int bn) __attribute__((always_inline)) {
    const int* rec = p.tile_tables + (long)bm * 8;
    const int f_lo = rec[0], f_hi = rec[1], e = rec[2];
    const unsigned long long mask = (unsigned long long)(unsigned)rec[3] | ((unsigned long long)(unsigned)rec[4] << 32);
    const int col_lo = bn * Cfg::BN;
    const int rows = f_hi - f_lo, cols = min(Cfg::BN, p.I - col_lo);
    if (p.do_wait) consumer_wait_or_produce(p.prod, mask, tid, Cfg::NTHREADS, &s_ticket);
    Out out;
    if constexpr (GATED) out = Out{p.y1 + (long)f_lo * (p.I / 2) + col_lo / 2, p.I / 2, p.act};
    else out = Out{p.y1 + (long)f_lo * p.I + col_lo, p.I};
    // row tiles of at most 64 rows: the deeper ring of the small tile shape (same thread count, same column range)
    if constexpr (kSmallShape) {
      if (rows <= Cfg64x256::BM) {
        moe_small_gather_tile<Out>(p.prod.gathered, p.H, p.sorted_row + f_lo, p.topk, p.w1 + (long)e * p.H * p.I + col_lo, p.I, out, rows, cols,
                                   p.H, smem);
        return;
      }
    }
    gemm_tile<Cfg, Out>(p.prod.gathered, p.H, p.sorted_row + f_lo, p.topk, p.w1 + (long)e * p.H * p.I + col_lo, p.I,
                        out, rows, cols, p.H, smem);
  };
  // the long tiles, in the usual order
  for (int pos = w; pos < sc.n_tiles; pos += sc.G) {
    int tile = sched_tile(sc, pos);
    int bi = tile / sc.nbn, bn = tile - bi * sc.nbn;
    do_tile(reorder ? s_perm[bi] : bi, bn);
  }
  // the short tiles: number j goes to one of the `idle` workgroups that the long tiles leave free in their last round
  // (two each), and beyond that to all workgroups in turn
  const int n_short = (n_rt - n_long) * p.nbn;
  const int used = sc.n_tiles % sc.G, idle = used ? sc.G - used : 0;
  for (int j = 0; reorder && j < n_short; j++) {
    int owner;
    if (j < 2 * idle) owner = used + j % idle;
    else owner = (j - 2 * idle) % sc.G;
    if (owner != w) continue;
    do_tile(s_perm[n_long + j / p.nbn], j % p.nbn);
  }
}

// ======================================================================================
// Part 2: grouped GEMM + scatter (+ gate weight) -> top-k reduce -> ReduceScatter.
//   stage A (GEMM tiles): Z[s,:] = w[row(s)] * (X2[s,:] . W2[e]) stored at scatter[row(s),:], row(s) = sorted_row[s];
//                         notifies counter (token block, column block) once per row it delivered there
//   stage B (top-k reduce tiles): waits for Tt*topk rows, partial[t,:] = sum_j scatter[t*topk+j,:], notifies the RS tile
//   stage C (RS tiles): the shared ReduceScatter consumer on `partial`
// ======================================================================================
template <bool WT>
struct ScatterRowsT {
  static constexpr bool SCALED = true, GATED = false;
  bf16_t* scatter;        // [T*topk, H] at the tile's first column
  long ld;
  const int* rows;        // sorted_row + f_lo
  const float* w;         // routing weights, flat [T*topk]
  __device__ __forceinline__ bf16_t* row(int r, float& scale) const {
    int rid = rows[r];
    scale = w[rid];
    return scatter + (long)rid * ld;
  }
  __device__ __forceinline__ void group(int /*r0*/) const {}
  // WT: written through to device scope, so that the tile's notification (RowsNotify) can follow a plain wait for these
  // stores; else ordinary stores, and the notification needs a release fence at device scope
  __device__ __forceinline__ void store(int r, int col, u32x4 v) const {
    if constexpr (WT) store16_device_scope(scatter + (long)rows[r] * ld + col, v); else *(u32x4*)(scatter + (long)rows[r] * ld + col) = v;
  }
};
typedef ScatterRowsT<true> ScatterRows;

struct MoeP2Params {
  const bf16_t* x2;         // [T*topk, I] sorted row order
  const bf16_t* w2;         // [E,I,H]
  bf16_t* scatter;          // [T*topk, H]
  const int* sorted_row;
  const int* tile_tables;
  const int* n_row_tiles;
  const float* topk_w;
  int T, H, I, topk;
  int nbn, G, swizzle;
  int Tt;                   // tokens per top-k reduce tile (= RS reduce tile rows)
  unsigned epoch;
  unsigned* rows_ready;     // [T/Tt * nbn] rows delivered per (token block, column block)
  RsSide rs;                // on partial [T,H]; rs.ready is raised by stage B
  int n_topk, n_rs;         // workgroups of stage B and C (in front of the grid when fused)
  int do_compute, do_notify, do_wait;
  int gb;  // column blocks walked side by side by stages A and B
};

__device__ void topk_reduce(const MoeP2Params& p, int wg, int n_wg, int tid, int nthreads) {
  const int ntb = p.T / p.Tt;
  const int n_tiles = ntb * p.nbn;
  const int BN = p.rs.Tn_r;
  for (int i = wg; i < n_tiles; i += n_wg) {
    // groups of column blocks slowest, like the GEMM stage that feeds it
    int tb, bn;
    colgroup_tile(i, ntb, p.nbn, p.gb, &tb, &bn);
    const int t_lo = tb * p.Tt, col_lo = bn * BN;
    const int cols = min(BN, p.H - col_lo);
    if (p.do_wait) {
      if (tid == 0) tile_wait(p.rows_ready + tb * p.nbn + bn, p.epoch * (unsigned)(p.Tt * p.topk), p.rs.ctl, tb * p.nbn + bn);
      __syncthreads();
    }
    // token t's routed rows are rows t*topk .. t*topk+topk-1 of the scatter buffer: source j = the buffer shifted by j rows, pitch topk*H
    const bf16_t* src0 = p.scatter + (long)t_lo * p.topk * p.H + col_lo;
    // a token block lies inside one rank's segment (Tt divides T/R): with direct push the reduced rows of another
    // rank's segment go straight to that rank's landing zone
    const int dest = t_lo / p.rs.seg_rows;
    bf16_t* dst = (!p.rs.direct || dest == p.rs.rank) ? p.rs.partial + (long)t_lo * p.H + col_lo
                                                      : p.rs.peer_push[dest] + (long)(t_lo - dest * p.rs.seg_rows) * p.H + col_lo;
    sum_tile<2, 2>([&](int j) { return src0 + (long)j * p.H; }, p.topk, dst, (long)p.topk * p.H, p.H, p.Tt, cols, tid, nthreads);
    wait_all_vmem();
    __syncthreads();   // every wave's written-through stores are complete: relaxed adds announce the tile
    if (tid == 0) {
      __hip_atomic_fetch_add(p.rs.ready + tb * p.rs.ncn + bn, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (producer_notifies_peer(p.rs, t_lo, p.Tt, col_lo, cols))   // final where it is: the owner hears of it at once
        __hip_atomic_fetch_add(p.rs.pushed + dest * p.rs.tiles_per_seg + (tb - dest * (p.rs.seg_rows / p.Tt)) * p.rs.ncn + bn, 1u,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// producer_tile_notify of one finished stage-A tile, with counts: the tile's rows are token-ascending, so every token
// block receives one run of them, and the first row of a run adds the run's length to the counter of (token block,
// column block).  Runs are found inside each wave of 64 rows with one ballot (a run that crosses a wave boundary is
// announced in two parts).  The tile's rows were stored written-through to device scope, so nothing but "every wave has
// seen its stores complete, and a workgroup barrier since" has to precede these relaxed adds: gemm_tile's hook provides
// that inside the NEXT tile's prologue, where the wait hides behind the latency of the first loads.
struct RowsNotify {
  const int* sorted_rows;   // sorted_row + f_lo of the tile
  unsigned* counters;       // rows_ready + column block
  int have, rows, topk, Tt, nbn;
  __device__ __forceinline__ bool pending() const { return have != 0; }
  __device__ __forceinline__ void run() const {
    const int r = threadIdx.x, lane = r & 63;
    const bool valid = r < rows;
    const int tb = valid ? (sorted_rows[r] / topk) / Tt : -1;
    const int prev = __shfl_up(tb, 1);
    const bool start = valid && (lane == 0 || prev != tb);
    const unsigned long long starts = __builtin_amdgcn_ballot_w64(start), valids = __builtin_amdgcn_ballot_w64(valid);
    if (start) {
      const unsigned long long later = lane == 63 ? 0ull : starts & ~((2ull << lane) - 1ull);
      const int end = later ? __builtin_ctzll(later) : __builtin_popcountll(valids);   // valid lanes are the low ones
      __hip_atomic_fetch_add(counters + (long)tb * nbn, (unsigned)(end - lane), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
};

// A row tile of at most 64 rows in the small tile shape with the deeper ring (see part 1).  Kept out of line: inlined
// beside the 256x256 loop it would raise the kernel's register count above what leaves room for the reduce kernel's
// waves on the same SIMDs.
__device__ __attribute__((noinline)) void moe_small_scatter_tile(const bf16_t* a, long lda, const bf16_t* b, long ldb, ScatterRows out, int rows,
                                                                 int cols, int K, char* smem, RowsNotify pend) {
  gemm_tile<Cfg64x256>(a, lda, nullptr, 1, b, ldb, out, rows, cols, K, smem, NoKWait{}, pend);
}

template <class Cfg>
__global__ void __launch_bounds__(Cfg::NTHREADS) moe_gemm_scatter_kernel(const MoeP2Params p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x;
  if ((int)blockIdx.x < p.n_topk) {
    topk_reduce(p, blockIdx.x, p.n_topk, tid, Cfg::NTHREADS);
    return;
  }
  if ((int)blockIdx.x < p.n_topk + p.n_rs) {
    rs_consumer(p.rs, blockIdx.x - p.n_topk, p.n_rs, tid, Cfg::NTHREADS);
    return;
  }
  if (!p.do_compute) return;
  __builtin_amdgcn_s_setprio(TL_COMPUTE_WAVE_PRIO);  // matrix waves go first when they share a SIMD with communication waves
  const int w = blockIdx.x - p.n_topk - p.n_rs;
  Sched sc;
  sc.nbm = *p.n_row_tiles;
  sc.nbn = p.nbn;
  sc.n_tiles = sc.nbm * sc.nbn;
  sc.G = p.G;
  sc.first_block = 0;
  sc.swizzle = p.swizzle;
  sc.group_m = 1;
  constexpr bool DEFER = Cfg::BN != 224;
  int have = 0, p_f_lo = 0, p_bn = 0, p_rows = 0;   // the previous tile of this workgroup awaits its notification
  for (int pos = w; pos < sc.n_tiles; pos += sc.G) {
    // groups of column blocks slowest: those columns of every token are complete early
    int bm, bn;
    colgroup_tile(sched_logical(sc, pos), sc.nbm, sc.nbn, p.gb, &bm, &bn);
    const int* rec = p.tile_tables + (long)bm * 8;
    const int f_lo = rec[0], f_hi = rec[1], e = rec[2];
    const int col_lo = bn * Cfg::BN;
    const int rows = f_hi - f_lo, cols = min(Cfg::BN, p.H - col_lo);
    bool small = false;
    if constexpr (Cfg::BM == 256 && Cfg::BN == 256) small = rows <= Cfg64x256::BM;
    // producer_tile_notify of the PREVIOUS tile happens inside this tile's prologue (RowsNotify); the 224-wide tile has
    // no register left for the state that carries from tile to tile and notifies right after its own stores
    const RowsNotify pend{p.sorted_row + p_f_lo, p.rows_ready + p_bn, DEFER ? have : 0, p_rows, p.topk, p.Tt, p.nbn};
    if (small)
      moe_small_scatter_tile(p.x2 + (long)f_lo * p.I, p.I, p.w2 + (long)e * p.I * p.H + col_lo, p.H,
                             ScatterRows{p.scatter + col_lo, p.H, p.sorted_row + f_lo, p.topk_w}, rows, cols, p.I, smem, pend);
    else if constexpr (DEFER)
      gemm_tile<Cfg>(p.x2 + (long)f_lo * p.I, p.I, nullptr, 1, p.w2 + (long)e * p.I * p.H + col_lo, p.H,
                     ScatterRows{p.scatter + col_lo, p.H, p.sorted_row + f_lo, p.topk_w}, rows, cols, p.I, smem, NoKWait{}, pend);
    else
      gemm_tile<Cfg>(p.x2 + (long)f_lo * p.I, p.I, nullptr, 1, p.w2 + (long)e * p.I * p.H + col_lo, p.H,
                     ScatterRowsT<false>{p.scatter + col_lo, p.H, p.sorted_row + f_lo, p.topk_w}, rows, cols, p.I, smem);
    if constexpr (DEFER) {
      if (p.do_notify) { have = 1; p_f_lo = f_lo; p_bn = bn; p_rows = rows; }
    } else if (p.do_notify) {
      __syncthreads();                                      // every wave's stores are complete ...
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // ... and written back to where every die sees them
      RowsNotify{p.sorted_row + f_lo, p.rows_ready + bn, 1, rows, p.topk, p.Tt, p.nbn}.run();
    }
  }
  if (have) {   // the last tile: nothing follows that could hide the wait for its stores
    wait_vmcnt<0>();
    __syncthreads();
    RowsNotify{p.sorted_row + p_f_lo, p.rows_ready + p_bn, 1, p_rows, p.topk, p.Tt, p.nbn}.run();
  }
}

// stages B and C as a kernel of their own (side-kernel binding)
// The top-k reduce workgroups join stage C when their own tiles are done: stage C hands its items out through a queue,
// and what becomes ready last (the last column group, at the very end) then spreads over all of them.
__global__ void __launch_bounds__(256) moe_reduce_kernel(const MoeP2Params p) {
  __shared__ int s_item;
  if ((int)blockIdx.x < p.n_topk) topk_reduce(p, blockIdx.x, p.n_topk, threadIdx.x, 256);
  rs_consumer(p.rs, blockIdx.x, gridDim.x, threadIdx.x, 256, &s_item);
}

__global__ void __launch_bounds__(256) moe_ag_producer_kernel(const AgProducer p) {
  __shared__ int s_ticket;
  ag_producer(p, threadIdx.x, 256, &s_ticket);
}

// ======================================================================================
// Host side
// ======================================================================================
struct MoeResolved {
  int variant, tile_m, tile_n, nbn, max_row_tiles;
  int G, n_comm;
  int Tm_p, Tn_p, n_ptm, n_ptn, rows_per_rank, rows_per_channel, expected;  // AllGather of the tokens (part 1)
  int Tt;                                                                     // top-k reduce / RS tile rows (part 2)
};

static int resolve_moe(const tl_ctx* ctx, int op, int T, int H, int I, int E, int topk, MoeResolved* r, bool paired_columns = false) {
  const tl_config& c = ctx->cfg;
  const int R = c.world_size;
  if (T <= 0 || H <= 0 || I <= 0 || E <= 0 || topk <= 0) return fail(TL_ERR_INVALID_ARG, "T, H, I, E, topk must be positive");
  if (E > kMaxExperts) return fail(TL_ERR_UNSUPPORTED_SHAPE, "at most %d experts (got %d)", kMaxExperts, E);
  if (topk > kMaxTopk || topk > E) return fail(TL_ERR_UNSUPPORTED_SHAPE, "topk=%d must be <= %d and <= E", topk, kMaxTopk);
  if (T % R) return fail(TL_ERR_UNSUPPORTED_SHAPE, "world size %d must divide T=%d", R, T);
  if ((T / R) % c.channels_per_rank) return fail(TL_ERR_UNSUPPORTED_SHAPE, "channels per rank %d must divide T/R=%d", c.channels_per_rank, T / R);
  if (R * c.channels_per_rank > 64) return fail(TL_ERR_UNSUPPORTED_SHAPE, "at most 64 AllGather channels (R*C=%d)", R * c.channels_per_rank);
  if (H % 64 || I % 64) return fail(TL_ERR_UNSUPPORTED_SHAPE, "H=%d and I=%d must be multiples of 64", H, I);
  // the grouped GEMM addresses a gathered token row as a 32-bit byte offset from the start of the token buffer
  if ((long)T * H * 2 >= (1L << 32)) return fail(TL_ERR_UNSUPPORTED_SHAPE, "the gathered token buffer (T*H = %ld elements) must stay below 4 GiB", (long)T * H);
  memset(r, 0, sizeof *r);
  const int N = (op == TL_OP_MOE_AG_GATHER_GEMM) ? I : H;
  int v = -1;
  if (c.tile_m || c.tile_n) {
    for (int i = 0; i < TILE_VARIANTS; i++)
      if (kTileM[i] == c.tile_m && kTileN[i] == c.tile_n) v = i;
    if (v < 0) return fail(TL_ERR_UNSUPPORTED_SHAPE, "compute tile %dx%d is not one of 256x256, 256x224, 128x128", c.tile_m, c.tile_n);
  } else if ((long)T * topk * N <= 1024L * 1024L) {
    v = TILE_128x128;
  } else {
    // 256x256 unless the 224-wide tile divides N and fills the last round of workgroups better; the number of
    // row tiles is data dependent: estimated as the routed rows over the tile height plus half a tile per expert
    auto fill = [&](int tn) {
      long tiles = ((long)T * topk / 256 + E / 2) * ceil_div(N, tn), G = ctx->num_cus;
      return (double)tiles * tn / (double)((tiles + G - 1) / G * G);
    };
    v = (!paired_columns && N % 224 == 0 && (N % 256 != 0 || fill(224) > 1.25 * fill(256))) ? TILE_256x224 : TILE_256x256;
  }
  if (paired_columns && v == TILE_256x224) return fail(TL_ERR_UNSUPPORTED_SHAPE, "the gated epilogue pairs 32-wide column blocks: the 256x224 tile has seven per wave");
  r->variant = v;
  r->tile_m = kTileM[v];
  r->tile_n = kTileN[v];
  r->nbn = ceil_div(N, r->tile_n);
  r->max_row_tiles = ceil_div(T * topk, r->tile_m) + E;
  r->G = c.compute_workgroups > 0 ? c.compute_workgroups : ctx->num_cus;
  // side kernels: one 256-thread workgroup fits on a compute unit beside a resident GEMM workgroup, and the reduce
  // stages of part 2 are bound by the bytes they keep in flight, so part 2 asks for one per compute unit
  r->n_comm = c.comm_workgroups > 0 ? c.comm_workgroups
                                    : (c.comm_mode == TL_COMM_WAVES ? 16 : (op == TL_OP_MOE_GEMM_SCATTER_RS ? 256 : 128));
  if (c.comm_mode == TL_COMM_NONE) r->n_comm = 0;
  r->rows_per_rank = T / R;
  r->rows_per_channel = r->rows_per_rank / c.channels_per_rank;
  int Tm_p = c.comm_tile_m;
  if (op == TL_OP_MOE_AG_GATHER_GEMM) {
    if (Tm_p == 0) {
      Tm_p = r->rows_per_channel;
      while (Tm_p > 32 && Tm_p % 2 == 0) Tm_p /= 2;
    }
    if (Tm_p <= 0 || r->rows_per_channel % Tm_p) return fail(TL_ERR_UNSUPPORTED_SHAPE, "producer row tile %d must divide T/(R*C)=%d", Tm_p, r->rows_per_channel);
    int Tn_p = c.comm_tile_n ? c.comm_tile_n : H;
    if (Tn_p <= 0 || H % Tn_p || Tn_p % 8) return fail(TL_ERR_UNSUPPORTED_SHAPE, "producer column tile %d must divide H=%d and be a multiple of 8", Tn_p, H);
    r->Tm_p = Tm_p; r->Tn_p = Tn_p; r->n_ptm = T / Tm_p; r->n_ptn = H / Tn_p;
    r->expected = (r->rows_per_channel / Tm_p) * r->n_ptn;
  } else {
    // every reduce tile ends with a notification (a device-scope release, microseconds): measured at T=8192, H=4096 the
    // fused call takes 0.67 / 0.51 / 0.45 / 0.42 / 0.44 ms with 32 / 64 / 128 / 256 / 512 tokens per tile
    int Tt = c.comm_tile_m;
    if (Tt == 0) {   // the largest divisor of T/R up to 128
      Tt = r->rows_per_rank >= 128 ? 128 : r->rows_per_rank;
      while (Tt > 1 && r->rows_per_rank % Tt) Tt--;
    }
    if (!c.comm_tile_m && r->rows_per_rank % 256 == 0 && (long)(T / 256) * r->nbn >= 2 * r->n_comm) Tt = 256;
    if (Tt <= 0 || r->rows_per_rank % Tt) return fail(TL_ERR_UNSUPPORTED_SHAPE, "top-k reduce tile of %d tokens must divide T/R=%d", Tt, r->rows_per_rank);
    if (H % r->tile_n) return fail(TL_ERR_UNSUPPORTED_SHAPE, "H=%d must be a multiple of the column tile %d", H, r->tile_n);
    r->Tt = Tt;
  }
  return TL_OK;
}

// LDS of the 256x256 kernels: they also hold the loop of the 64-row tile shape
constexpr int kLds256 = Cfg256x256::LDS_BYTES > Cfg64x256::LDS_BYTES ? Cfg256x256::LDS_BYTES : Cfg64x256::LDS_BYTES;
static_assert(Cfg64x256::NTHREADS == Cfg256x256::NTHREADS && Cfg64x256::BN == Cfg256x256::BN, "the two shapes share workgroup and column range");

template <class P>
static int launch_moe(int variant, void (*k0)(const P), void (*k1)(const P), void (*k2)(const P), const P& p, int grid, hipStream_t s,
                      int lds256 = Cfg256x256::LDS_BYTES) {
  switch (variant) {
    case TILE_256x256: return launch_fused<Cfg256x256>(k0, p, grid, s, lds256);
    case TILE_256x224: return launch_fused<Cfg256x224>(k1, p, grid, s);
    default: return launch_fused<Cfg128x128>(k2, p, grid, s);
  }
}

}  // namespace tl

using namespace tl;

extern "C" {

int tl_moe_query(const tl_ctx* ctx, int op, int T, int H, int I, int E, int topk, int* info) {
  if (int e = check_ctx(ctx)) return e;
  if (!info) return fail(TL_ERR_INVALID_ARG, "info must not be null");
  if (op != TL_OP_MOE_AG_GATHER_GEMM && op != TL_OP_MOE_GEMM_SCATTER_RS) return fail(TL_ERR_INVALID_ARG, "tl_moe_query: operator %d is not a MoE half", op);
  MoeResolved r;
  if (int e = resolve_moe(ctx, op, T, H, I, E, topk, &r)) return e;
  const int R = ctx->cfg.world_size;
  int n_flags;
  if (op == TL_OP_MOE_AG_GATHER_GEMM) n_flags = R * ctx->cfg.channels_per_rank;
  else {
    int ntb = T / r.Tt, tps = (T / R / r.Tt) * r.nbn;
    n_flags = ntb * r.nbn /*rows_ready*/ + ntb * r.nbn /*rs ready*/ + 2 * R * tps;
  }
  int v[8] = {r.tile_m, r.tile_n, r.max_row_tiles, n_flags, 256, r.expected, r.Tt, r.nbn};
  memcpy(info, v, sizeof v);
  return TL_OK;
}

int tl_moe_route(tl_ctx* ctx, const float* gate_logits, int T, int E, int topk, int renormalize, int tile_m, int* topk_ids, float* topk_w,
                 int* expert_offsets, int* sorted_row, int* tile_tables, int* n_tiles, void* stream) {
  if (int e = check_op_ctx(ctx)) return e;
  if (!gate_logits || !topk_ids || !topk_w || !expert_offsets || !sorted_row || !tile_tables || !n_tiles) return fail(TL_ERR_INVALID_ARG, "tl_moe_route: null pointer argument");
  const tl_config& c = ctx->cfg;
  if (T <= 0 || E <= 0 || topk <= 0 || tile_m <= 0) return fail(TL_ERR_INVALID_ARG, "tl_moe_route: T, E, topk, tile_m must be positive");
  if (E > kMaxExperts || topk > kMaxTopk || topk > E) return fail(TL_ERR_UNSUPPORTED_SHAPE, "tl_moe_route: E <= %d, topk <= %d and topk <= E required", kMaxExperts, kMaxTopk);
  if (T % c.world_size || (T / c.world_size) % c.channels_per_rank) return fail(TL_ERR_UNSUPPORTED_SHAPE, "tl_moe_route: R must divide T and C must divide T/R");
  if (c.world_size * c.channels_per_rank > 64) return fail(TL_ERR_UNSUPPORTED_SHAPE, "tl_moe_route: at most 64 AllGather channels");
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(moe_topk_kernel, dim3((T + 255) / 256), dim3(256), 0, s, gate_logits, T, E, topk, renormalize, topk_ids, topk_w);
  TL_HIP(hipGetLastError());
  hipLaunchKernelGGL(moe_sort_kernel, dim3(1), dim3(kRouteThreads), 0, s, topk_ids, T * topk, E, topk, T, c.world_size, c.channels_per_rank,
                     tile_m, expert_offsets, sorted_row, tile_tables, n_tiles);
  TL_HIP(hipGetLastError());
  return TL_OK;
}

static int moe_p1_impl(tl_ctx* ctx, const void* const* x_shards, void* x_gathered, const void* w1, const int* sorted_row,
                       const int* tile_tables, const int* n_tiles, void* y1, int T, int H, int I, int E, int topk, int act, unsigned* flags,
                       unsigned epoch, void* workspace, size_t ws_bytes, void* compute_stream, void* comm_stream) {
  if (int e = check_op_ctx(ctx)) return e;
  const tl_config& cfg = ctx->cfg;
  if (!x_shards || !x_gathered || !w1 || !sorted_row || !tile_tables || !n_tiles || !y1 || !flags || !workspace)
    return fail(TL_ERR_INVALID_ARG, "tl_moe_ag_gather_gemm: null pointer argument");
  if (epoch == 0) return fail(TL_ERR_INVALID_ARG, "tl_moe_ag_gather_gemm: epoch starts at 1");
  MoeResolved r;
  if (int e = resolve_moe(ctx, TL_OP_MOE_AG_GATHER_GEMM, T, H, I, E, topk, &r, act != 0)) return e;
  if (ws_bytes < 256) return fail(TL_ERR_WORKSPACE_TOO_SMALL, "tl_moe_ag_gather_gemm: workspace of %zu bytes, 256 needed", ws_bytes);
  for (int q = 0; q < cfg.world_size; q++)
    if (!x_shards[q] || !aligned16(x_shards[q])) return fail(TL_ERR_INVALID_ARG, "tl_moe_ag_gather_gemm: x_shards[%d] is null or misaligned", q);
  if (!aligned16(x_gathered) || !aligned16(w1) || !aligned16(y1)) return fail(TL_ERR_INVALID_ARG, "tl_moe_ag_gather_gemm: device pointers must be 16-byte aligned");
  if (cfg.comm_mode == TL_COMM_STREAM || cfg.comm_mode == TL_COMM_EXTERNAL || cfg.comm_mode == TL_COMM_COPY_ENGINE)
    return fail(TL_ERR_INVALID_ARG, "tl_moe_ag_gather_gemm: comm_mode must be NONE, WAVES or SIDE_KERNEL");

  MoeP1Params p;
  memset(&p, 0, sizeof p);
  fill_ag_producer(ctx, &p.prod, x_shards, x_gathered, H, r.Tm_p, r.Tn_p, r.n_ptm, r.n_ptn, r.rows_per_rank, r.rows_per_channel, flags,
                   epoch, workspace);
  p.prod.wait_target = epoch * (unsigned)r.expected;
  p.w1 = (const bf16_t*)w1;
  p.y1 = (bf16_t*)y1;
  p.sorted_row = sorted_row;
  p.tile_tables = tile_tables;
  p.n_row_tiles = n_tiles;
  p.H = H; p.I = I; p.topk = topk;
  p.act = act;
  p.nbn = r.nbn; p.G = r.G; p.swizzle = cfg.xcd_swizzle;
  p.group_m = cfg.group_m > 0 ? cfg.group_m : 4;
  hipStream_t cs = (hipStream_t)compute_stream, ms = (hipStream_t)comm_stream;
  const bool alone = cfg.comm_alone != 0;
  p.do_compute = alone ? 0 : 1;
  auto launch = [&](int grid) {
    if (act) {
      if (r.variant == TILE_256x256) return launch_fused<Cfg256x256>(moe_ag_gather_gemm_kernel<Cfg256x256, true>, p, grid, cs, kLds256);
      return launch_fused<Cfg128x128>(moe_ag_gather_gemm_kernel<Cfg128x128, true>, p, grid, cs);
    }
    return launch_moe<MoeP1Params>(r.variant, moe_ag_gather_gemm_kernel<Cfg256x256>, moe_ag_gather_gemm_kernel<Cfg256x224>,
                                   moe_ag_gather_gemm_kernel<Cfg128x128>, p, grid, cs, kLds256);
  };
  switch (cfg.comm_mode) {
    case TL_COMM_NONE:
      if (alone) return fail(TL_ERR_INVALID_ARG, "tl_moe_ag_gather_gemm: comm_alone needs a producer");
      p.n_comm = 0; p.do_wait = 0;
      return launch(r.G);
    case TL_COMM_WAVES:
      p.n_comm = r.n_comm; p.do_wait = 1;
      return launch(alone ? r.n_comm : r.G + r.n_comm);
    case TL_COMM_SIDE_KERNEL:
      p.n_comm = 0; p.do_wait = 1;
      hipLaunchKernelGGL(moe_ag_producer_kernel, dim3(r.n_comm), dim3(256), 0, ms, p.prod);
      TL_HIP(hipGetLastError());
      return alone ? TL_OK : launch(r.G);
  }
  return fail(TL_ERR_INVALID_ARG, "tl_moe_ag_gather_gemm: unknown comm_mode");
}

int tl_moe_ag_gather_gemm(tl_ctx* ctx, const void* const* x_shards, void* x_gathered, const void* w1, const int* sorted_row,
                          const int* tile_tables, const int* n_tiles, void* y1, int T, int H, int I, int E, int topk, unsigned* flags,
                          unsigned epoch, void* workspace, size_t ws_bytes, void* compute_stream, void* comm_stream) {
  return moe_p1_impl(ctx, x_shards, x_gathered, w1, sorted_row, tile_tables, n_tiles, y1, T, H, I, E, topk, 0, flags, epoch, workspace, ws_bytes,
                     compute_stream, comm_stream);
}

int tl_moe_ag_gather_gemm_act_mul(tl_ctx* ctx, const void* const* x_shards, void* x_gathered, const void* w1_gate_up, const int* sorted_row,
                                  const int* tile_tables, const int* n_tiles, void* y1, int T, int H, int F, int E, int topk, int act,
                                  unsigned* flags, unsigned epoch, void* workspace, size_t ws_bytes, void* compute_stream, void* comm_stream) {
  if (act != TL_ACT_SILU_MUL && act != TL_ACT_GELU_MUL) return fail(TL_ERR_INVALID_ARG, "tl_moe_ag_gather_gemm_act_mul: unknown activation %d", act);
  if (F <= 0 || F > (1 << 29)) return fail(TL_ERR_INVALID_ARG, "tl_moe_ag_gather_gemm_act_mul: F=%d out of range", F);
  if (F % 32) return fail(TL_ERR_UNSUPPORTED_SHAPE, "tl_moe_ag_gather_gemm_act_mul: F=%d is not a multiple of 32 (gate and up alternate in blocks of 32 columns)", F);
  return moe_p1_impl(ctx, x_shards, x_gathered, w1_gate_up, sorted_row, tile_tables, n_tiles, y1, T, H, 2 * F, E, topk, act, flags, epoch, workspace,
                     ws_bytes, compute_stream, comm_stream);
}

int tl_moe_gemm_scatter_rs(tl_ctx* ctx, const void* x2, const void* w2, const int* sorted_row, const int* tile_tables, const int* n_tiles,
                           const float* topk_w, void* scatter_buf, void* partial, const void* const* peer_recv, void* const* peer_push,
                           void* out, int T, int H, int I, int E, int topk, unsigned* flags, unsigned epoch, void* workspace,
                           size_t ws_bytes, void* compute_stream, void* comm_stream) {
  if (int e = check_op_ctx(ctx)) return e;
  const tl_config& cfg = ctx->cfg;
  if (!x2 || !w2 || !sorted_row || !tile_tables || !n_tiles || !topk_w || !scatter_buf || !partial || !peer_recv || !peer_push || !out || !flags || !workspace)
    return fail(TL_ERR_INVALID_ARG, "tl_moe_gemm_scatter_rs: null pointer argument");
  if (epoch == 0) return fail(TL_ERR_INVALID_ARG, "tl_moe_gemm_scatter_rs: epoch starts at 1");
  MoeResolved r;
  if (int e = resolve_moe(ctx, TL_OP_MOE_GEMM_SCATTER_RS, T, H, I, E, topk, &r)) return e;
  if (ws_bytes < 256) return fail(TL_ERR_WORKSPACE_TOO_SMALL, "tl_moe_gemm_scatter_rs: workspace of %zu bytes, 256 needed", ws_bytes);
  const int R = cfg.world_size;
  if (!aligned16(x2) || !aligned16(w2) || !aligned16(scatter_buf) || !aligned16(partial) || !aligned16(out))
    return fail(TL_ERR_INVALID_ARG, "tl_moe_gemm_scatter_rs: device pointers must be 16-byte aligned");
  for (int q = 0; q < R; q++)
    if (q != cfg.rank && (!peer_recv[q] || !peer_push[q] || !aligned16(peer_recv[q]) || !aligned16(peer_push[q])))
      return fail(TL_ERR_INVALID_ARG, "tl_moe_gemm_scatter_rs: peer_recv[%d] or peer_push[%d] is null or misaligned", q, q);
  if (cfg.comm_mode == TL_COMM_STREAM || cfg.comm_mode == TL_COMM_EXTERNAL || cfg.comm_mode == TL_COMM_COPY_ENGINE)
    return fail(TL_ERR_INVALID_ARG, "tl_moe_gemm_scatter_rs: comm_mode must be NONE, WAVES or SIDE_KERNEL");

  MoeP2Params p;
  memset(&p, 0, sizeof p);
  p.x2 = (const bf16_t*)x2; p.w2 = (const bf16_t*)w2; p.scatter = (bf16_t*)scatter_buf;
  p.sorted_row = sorted_row; p.tile_tables = tile_tables; p.n_row_tiles = n_tiles; p.topk_w = topk_w;
  p.T = T; p.H = H; p.I = I; p.topk = topk;
  p.nbn = r.nbn; p.G = r.G; p.swizzle = cfg.xcd_swizzle;
  p.Tt = r.Tt;
  // measured at T=8192, H=4096, I=1792: the wider the group the better (fused 0.59 ms at 1, 0.50 ms at 16): the stages
  // gain little from running side by side, and narrow groups concentrate the traffic on few memory channels
  p.gb = cfg.group_m > 0 ? cfg.group_m : 16;
  if (p.gb > r.nbn) p.gb = r.nbn;
  p.epoch = epoch;
  const int ntb = T / r.Tt;
  p.rows_ready = flags;
  // stage B raises one notification per reduce tile: for the RS consumer the "producer tile" is the reduce tile itself
  fill_rs_side(ctx, &p.rs, partial, peer_recv, peer_push, out, T, H, r.Tt, r.tile_n, r.Tt, r.tile_n, flags + (size_t)ntb * r.nbn, epoch, workspace);
  if (cfg.tile_order != TL_ORDER_NATURAL) {
    int first = cfg.tile_order >= TL_ORDER_OWN_FIRST ? cfg.rank : (cfg.rank + 1) % R;
    p.rs.rs_first_block = first * (T / R / r.Tt);
  }
  if (p.rs.direct == 2) p.rs.direct = 1;  // the own segment is reduced by stage C here (stage B has no peer data at hand)
  if (!aligned128(scatter_buf)) p.rs.ctl.strict = 1;  // stage B's guarded regions are column blocks of the scatter buffer
  hipStream_t cs = (hipStream_t)compute_stream, ms = (hipStream_t)comm_stream;
  const bool alone = cfg.comm_alone != 0;
  p.do_compute = alone ? 0 : 1;
  auto launch = [&](int grid) {
    return launch_moe<MoeP2Params>(r.variant, moe_gemm_scatter_kernel<Cfg256x256>, moe_gemm_scatter_kernel<Cfg256x224>,
                                   moe_gemm_scatter_kernel<Cfg128x128>, p, grid, cs, kLds256);
  };
  // split of the communication workgroups between stage B (top-k reduce: topk reads per output tile) and stage C
  // (ReduceScatter).  Without direct push C reads and writes every tile once more: even split.  With direct push C
  // only reduces the own segment, but that is R reads per tile for 1/R of the tiles: still a third of all reads.
  int n_rs = cfg.rs_direct_push && r.n_comm >= 8 ? r.n_comm * 3 / 8 : r.n_comm / 2;
  if (n_rs < 1) n_rs = 1;
  const int n_topk = r.n_comm - n_rs > 0 ? r.n_comm - n_rs : 1;
  switch (cfg.comm_mode) {
    case TL_COMM_NONE:
      if (alone) return fail(TL_ERR_INVALID_ARG, "tl_moe_gemm_scatter_rs: comm_alone needs a comm_mode with a reduce side");
      p.n_topk = 0; p.n_rs = 0; p.do_notify = 0;
      return launch(r.G);
    case TL_COMM_WAVES:
      if (int e = launch_peers_arrive(p.rs, alone ? cs : ms)) return e;
      p.n_topk = n_topk; p.n_rs = n_rs; p.do_notify = alone ? 0 : 1; p.do_wait = alone ? 0 : 1;
      return launch(alone ? n_topk + n_rs : r.G + n_topk + n_rs);
    case TL_COMM_SIDE_KERNEL:
      p.n_topk = 0; p.n_rs = 0; p.do_notify = alone ? 0 : 1; p.do_wait = alone ? 0 : 1;
      if (!alone)
        if (int e = launch(r.G)) return e;
      if (int e = launch_peers_arrive(p.rs, ms)) return e;
      p.n_topk = n_topk; p.n_rs = n_rs;
      use_rs_queue(&p.rs, workspace, epoch);   // (stage A above was given its parameters by value before this)
      hipLaunchKernelGGL(moe_reduce_kernel, dim3(n_topk + n_rs), dim3(256), 0, ms, p);
      TL_HIP(hipGetLastError());
      return TL_OK;
  }
  return fail(TL_ERR_INVALID_ARG, "tl_moe_gemm_scatter_rs: unknown comm_mode");
}

}  // extern "C"
