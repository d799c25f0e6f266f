// ReduceScatter side shared by GEMM+RS and the MoE second half: reduce tiles of a partial result,
// their ready / peer counters, and the consumer that reduces the own segment and pushes the others.
#pragma once
#include "tl_device.h"

namespace tl {

struct RsSide {
  bf16_t* partial;                  // [M,N] local partial result (written by the producer stage)
  const bf16_t* peer_recv[kMaxWorld];
  bf16_t* peer_push[kMaxWorld];
  bf16_t* out;                      // [M/R,N]
  int M, N, R, rank;
  int tile_m, tile_n;               // tile of the producer stage (decides how many notifications a reduce tile expects)
  int Tm_r, Tn_r, ncm, ncn;         // reduce tiles
  int seg_rows, tiles_per_seg;
  int rs_first_block;               // rotation of reduce row-blocks
  int do_wait;                      // wait for the producer stage's notifications
  int direct;                       // 1: the producer stage stored the other segments' rows into peer_push itself;
                                    // 2: it also reduced the own segment in its epilogue (the consumer only forwards)
  int fast_rows;                    // a segment of the partial result spans less than 4 GiB: 32-bit offsets inside it
  int ring;                         // ring ReduceScatter: peer_recv[q] = the next rank's running sum of segment q,
                                    // peer_push[q] = the previous rank's landing zone for this rank's running sum of it
  unsigned epoch;
  unsigned* ready;                  // [ncm*ncn]
  unsigned* arrived;                // [R*tiles_per_seg]
  unsigned* pushed;                 // [R*tiles_per_seg]
  int slices;                       // >= 1: a reduce tile of the own segment is handed out in this many row slices
  int others_done;                  // 1: every reduce tile of another segment is announced by its producer (direct push, each
                                    // reduce tile inside one producer tile): the reduce side has items of the own segment only
  unsigned* queue;                  // head of the work-item queue of the reduce side (word 1 of the workspace: it grows by the
                                    // call's number of items), or null: items are dealt out by workgroup index
  unsigned queue_end;               // epoch * items per call
  WaitCtl ctl;
};

// With direct push a reduce tile of another rank's segment is final once the producer stage has stored it.  When one
// producer tile covers the whole reduce tile, the producer's own notification can therefore tell the owner as well
// (peer_tile_notify straight from the producer), and the consumer has nothing left to do for that tile; tiles that
// several producer tiles share still go through the consumer, which waits for all of them.
__device__ __forceinline__ bool producer_notifies_peer(const RsSide& p, int row_lo, int rows, int col_lo, int cols) {
  if (!p.direct || p.ring || !p.do_wait) return false;
  if (row_lo / p.seg_rows == p.rank) return false;
  return (row_lo + rows - 1) / p.tile_m == row_lo / p.tile_m && (col_lo + cols - 1) / p.tile_n == col_lo / p.tile_n;
}

// ======================================================================================
// ReduceScatter consumer: reduce tiles of the partial product.  Own segment: wait for every
// peer's rows, sum in fp32 in rank order, store bf16.  Other segments: push to the owner's
// landing zone and notify it.
// ======================================================================================
// Work items of the reduce side.  A reduce tile of the own segment is the heavy kind -- R sources of tile size read by
// one workgroup, which is bound by the bytes it keeps in flight -- and needs no notification afterwards: each of its
// p.slices row slices is an item, so that the tiles that become ready last (in MoE part 2: a whole column group at the
// very end) spread over all workgroups of the reduce side.  Every tile of another segment is one item, unless its
// producer announces it itself (others_done).  The items of the own segment come first if the visiting order starts with
// it, else last; inside each kind the visiting order holds, which is the order in which the tiles become ready.  The ring
// form has one item per tile in visiting order.
__host__ __device__ inline int rs_item_count(const RsSide& p) {
  const int n_rt = p.ncm * p.ncn, own = (p.seg_rows / p.Tm_r) * p.ncn;
  if (p.ring) return n_rt;
  return own * p.slices + (p.others_done ? 0 : n_rt - own);
}

// With a queue the items go to whoever asks next; workgroups that had other work first (stage B of MoE part 2) join when
// they are done.  s_item: an int in LDS for handing the claimed item to the workgroup.
__device__ void rs_consumer(const RsSide& p, int wg, int n_wg, int tid, int nthreads, int* s_item = nullptr) {
  const int n_rt = p.ncm * p.ncn;
  const int cm_per_seg = p.seg_rows / p.Tm_r;
  const int S = p.ring ? 1 : p.slices;
  const int n_items = rs_item_count(p);
  const int n_own = p.ring ? 0 : cm_per_seg * p.ncn * S, n_oth = n_items - n_own;
  const int own_lo = p.rank * cm_per_seg;                                   // first row block of the own segment
  int own_rel = own_lo - p.rs_first_block;                                  // ... and its place in the visiting order
  if (own_rel < 0) own_rel += p.ncm;
  const bool own_first = own_rel == 0;
  const bool queued = p.queue != nullptr && s_item != nullptr;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int it = wg;; it += n_wg) {
    if (queued) {
      if (wave == 0) {
        const unsigned t = lane0_fetch_add(p.queue, 1u);
        const unsigned idx = t - (p.queue_end - (unsigned)n_items);
        if (idx >= (unsigned)n_items) lane0_add(p.queue, 0xffffffffu);   // past the end (or not this epoch's counter): give it back
        *s_item = idx < (unsigned)n_items ? (int)idx : -1;
      }
      __syncthreads();
      it = __builtin_amdgcn_readfirstlane(*s_item);
      __syncthreads();
      if (it < 0) break;
    } else if (it >= n_items) break;
    int cm, cn, slice = 0;
    if (p.ring) {
      const int cmi = it / p.ncn;
      cn = it - cmi * p.ncn;
      cm = cmi + p.rs_first_block;
      if (cm >= p.ncm) cm -= p.ncm;
    } else {
      const bool own = own_first ? it < n_own : it >= n_oth;
      if (own) {
        const int j = own_first ? it : it - n_oth;
        const int tl_ = j / S;
        slice = j - tl_ * S;
        cm = own_lo + tl_ / p.ncn;
        cn = tl_ % p.ncn;
      } else {
        const int j = own_first ? it - n_own : it;
        const int k = j / p.ncn;                       // k-th row block of another segment in visiting order
        cn = j - k * p.ncn;
        cm = p.rs_first_block + (k < own_rel ? k : k + cm_per_seg);
        if (cm >= p.ncm) cm -= p.ncm;
      }
    }
    const int t = cm * p.ncn + cn;
    const int tile_row_lo = cm * p.Tm_r, col_lo = cn * p.Tn_r;
    const int tile_rows = min(p.Tm_r, p.M - tile_row_lo), cols = min(p.Tn_r, p.N - col_lo);
    const int dest = tile_row_lo / p.seg_rows;                  // owner of these rows in the scattered output
    const int local = (cm - dest * cm_per_seg) * p.ncn + cn;    // reduce-tile index inside its segment
    // the rows of this item: a slice of an own-segment tile, else the whole tile
    int row_lo = tile_row_lo, rows = tile_rows;
    if (S > 1 && dest == p.rank) {
      const int per = (tile_rows + S - 1) / S;
      row_lo = tile_row_lo + slice * per;
      rows = min(per, tile_row_lo + tile_rows - row_lo);
      if (rows <= 0) continue;
    }
    const int seg_row = row_lo - dest * p.seg_rows;
    if (p.ring) {
      // Ring order (paper: kernel design, GEMM + ring ReduceScatter): the running sum of segment q travels from rank
      // q-1 down to rank q.  This rank starts the chain of segment rank+1 (its partial rows go on unchanged), adds its
      // partial rows to what the next rank passed on for every other segment, and hands the sum to the previous rank --
      // or, for its own segment, the last hop, stores it as the result.
      const int start = p.rank + 1 == p.R ? 0 : p.rank + 1;
      if (tid == 0) {
        if (p.do_wait) {
          unsigned n_m = (unsigned)((tile_row_lo + tile_rows - 1) / p.tile_m - tile_row_lo / p.tile_m + 1);
          unsigned n_n = (unsigned)((col_lo + cols - 1) / p.tile_n - col_lo / p.tile_n + 1);
          tile_wait(p.ready + t, p.epoch * n_m * n_n, p.ctl, t);                                    // consumer_tile_wait
        }
        if (dest != start) tile_wait(p.arrived + dest * p.tiles_per_seg + local, p.epoch, p.ctl, n_rt + dest * p.tiles_per_seg + local);  // peer_tile_wait
      }
      __syncthreads();
      const long seg_off = (long)seg_row * p.N + col_lo;
      const bf16_t* own = p.partial + (long)row_lo * p.N + col_lo;
      bf16_t* dst = (dest == p.rank ? p.out : p.peer_push[dest]) + seg_off;
      if (dest == start) {   // chain start (in a world of one rank also the last hop: dst is the result)
        copy_tile(own, p.N, dst, p.N, rows, cols, tid, nthreads);
      } else {
        const bf16_t* inc = p.peer_recv[dest] + seg_off;
        sum_tile<2, 2>([&](int j) { return j == 0 ? own : inc; }, 2, dst, p.N, p.N, rows, cols, tid, nthreads);
      }
      if (dest != p.rank) {
        wait_all_vmem();
        __syncthreads();   // every wave's written-through stores are complete
        if (tid == 0) notify_relaxed(p.pushed + dest * p.tiles_per_seg + local);                      // peer_tile_notify
      }
      continue;
    }
    if (p.direct == 2 && dest == p.rank) continue;  // reduced by the producer stage's epilogue
    if (producer_notifies_peer(p, tile_row_lo, tile_rows, col_lo, cols)) continue;
    // the waits of one item side by side, one lane each: lane 0 consumer_tile_wait (all GEMM tiles that overlap this
    // reduce tile have stored their part), lane 1 + q peer_tile_wait for peer q's contribution to a tile of the own segment
    if (tid == 0) {
      if (p.do_wait) {
        unsigned n_m = (unsigned)((tile_row_lo + tile_rows - 1) / p.tile_m - tile_row_lo / p.tile_m + 1);
        unsigned n_n = (unsigned)((col_lo + cols - 1) / p.tile_n - col_lo / p.tile_n + 1);
        tile_wait(p.ready + t, p.epoch * n_m * n_n, p.ctl, t);
      }
    } else if (tid <= p.R && dest == p.rank) {
      const int q = tid - 1;
      if (q != p.rank) tile_wait(p.arrived + q * p.tiles_per_seg + local, p.epoch, p.ctl, n_rt + q * p.tiles_per_seg + local);
    }
    __syncthreads();
    const bf16_t* mine = p.partial + (long)row_lo * p.N + col_lo;
    if (dest == p.rank) {
      const long seg_off = (long)seg_row * p.N + col_lo;
      sum_tile<4>([&](int q) { return q == p.rank ? mine : p.peer_recv[q] + seg_off; }, p.R, p.out + seg_off, p.N, p.N, rows, cols, tid,
               nthreads);
    } else {
      // tile_push_data to the owner's landing zone (unless the producer stage has put the rows there itself), then
      // peer_tile_notify
      if (!p.direct) copy_tile(mine, p.N, p.peer_push[dest] + (long)seg_row * p.N + col_lo, p.N, rows, cols, tid, nthreads);
      wait_all_vmem();
      __syncthreads();   // every wave's written-through stores are complete (with direct push: the producer's already were)
      if (tid == 0) notify_relaxed(p.pushed + dest * p.tiles_per_seg + local);
    }
  }
}


// Where the rows of a [M,N] partial result go (output functor of the matrix tile): row g of the own segment to
// partial[g,:], and with direct push row g of segment q to peer_push[q][g - q*seg_rows,:]; else all rows to partial.
// WT: the rows are stored written-through to device scope, so that the tile's notification can follow a plain wait for
// the stores (TileNotify); else ordinary stores, and the notification needs a release fence at device scope.
//
// The destination depends on the row's segment.  One store instruction of the tile's epilogue covers a few consecutive
// rows, and the functor remembers the segment [seg_lo, seg_hi) of the last group's first row with the base address of its
// destination: a group that lies in that segment is stored as (scalar base) + (32-bit lane offset) with no per-lane
// segment arithmetic; only lanes of a group that straddles a segment boundary take the per-lane path.
// FAST = false: always the per-lane path (for a tile shape that has no register left for the remembered segment).
template <bool WT, bool FAST = true>
struct PushRowsT {
  static constexpr bool SCALED = false, GATED = false;
  const RsSide* rs;
  int row_lo, col_lo;
  int seg_lo = 0, seg_hi = 0;       // global rows of the remembered segment (empty: nothing remembered yet)
  const bf16_t* seg_base = nullptr; // address of row seg_lo, column col_lo, of that segment's destination
  __device__ __forceinline__ bf16_t* row(int r, float& scale) const {
    const int g = row_lo + r;
    const int dest = g / rs->seg_rows;
    if (!rs->direct || dest == rs->rank) return rs->partial + (long)g * rs->N + col_lo;
    return rs->peer_push[dest] + (long)(g - dest * rs->seg_rows) * rs->N + col_lo;
  }
  // r0 = first row of the next instruction's group of rows; every lane calls this, in uniform control flow
  __device__ __forceinline__ void group(int r0) {
    if (!FAST || rs->direct == 2 || !rs->fast_rows) return;
    const int g0 = __builtin_amdgcn_readfirstlane(row_lo + r0);
    if (g0 < seg_lo || g0 >= seg_hi) {   // uniform: a new segment starts (once or twice per tile)
      const int dest = __builtin_amdgcn_readfirstlane(g0 / rs->seg_rows);
      seg_lo = dest * rs->seg_rows;
      seg_hi = seg_lo + rs->seg_rows;
      const bf16_t* b = (!rs->direct || dest == rs->rank) ? rs->partial + (long)seg_lo * rs->N + col_lo : rs->peer_push[dest] + col_lo;
      seg_base = (const bf16_t*)uniform64((unsigned long long)b);
    }
  }
  // 8 values of tile row r at tile column col
  __device__ __forceinline__ void store(int r, int col, u32x4 v) const {
    const int g = row_lo + r;
    if (FAST && rs->direct != 2 && rs->fast_rows) {
      if (g < seg_hi) {
        const unsigned off = ((unsigned)(g - seg_lo) * (unsigned)rs->N + (unsigned)col) * 2u;
        if constexpr (WT) store16_device_scope(seg_base, off, v); else *(u32x4*)((char*)seg_base + off) = v;
        return;
      }
    }
    store_lane(g, col, v);
  }
  // Per-lane path.  Mode 2, own segment: besides the bf16 partial, out = bf16(sum over ranks in rank order, fp32) with
  // the R-1 peer values of the same place loaded together (the caller has done the peer_tile_wait): the same arithmetic
  // as the consumer's sum, so both paths give identical bits.
  __device__ __forceinline__ void store_lane(int g, int col, u32x4 v) const {
    const int dest = g / rs->seg_rows;
    if (!rs->direct || dest == rs->rank) {
      put(rs->partial + (long)g * rs->N + col_lo + col, v);
      if (rs->direct == 2) {
        const long off = (long)(g - dest * rs->seg_rows) * rs->N + col_lo + col;
        u32x4 pv[kMaxWorld];
#pragma unroll
        for (int q = 0; q < kMaxWorld; q++)
          if (q < rs->R && q != rs->rank) pv[q] = __builtin_nontemporal_load((const u32x4*)(rs->peer_recv[q] + off));
        float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < kMaxWorld; q++)
          if (q < rs->R) acc_bf16x8(s, q == rs->rank ? v : pv[q]);
        *(u32x4*)(rs->out + off) = pack_bf16x8(s);
      }
    } else {
      put(rs->peer_push[dest] + (long)(g - dest * rs->seg_rows) * rs->N + col_lo + col, v);
    }
  }
  __device__ __forceinline__ void put(bf16_t* p, u32x4 v) const {
    if constexpr (WT) store16_device_scope(p, v); else *(u32x4*)p = v;
  }
};

// Simulated peers: peer q's push of every tile of this rank's segment "arrives".
__global__ void peers_arrive_kernel(unsigned* arrived, int tiles_per_seg, int R, int rank);

}  // namespace tl
