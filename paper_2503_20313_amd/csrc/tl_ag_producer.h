// AllGather side shared by the operators that gather row shards (AG+GEMM, AG+gather+grouped GEMM):
// producer-tile queue, producers, and the consumer wait that helps producing.  gfx950 only.
#pragma once
#include "tl_device.h"

namespace tl {

struct AgProducer {
  const bf16_t* shards[kMaxWorld];  // shard q = rows [q*rows_per_rank, (q+1)*rows_per_rank), each [rows_per_rank, ld]
  bf16_t* gathered;                 // [R*rows_per_rank, ld]
  int ld;                           // row length in elements (K of AG+GEMM, H of the MoE token buffer)
  int R, rank;
  int first_src;                    // source rank whose tiles head the queue; the queue then follows the ring
  int n_ptm_all;                    // row tiles of the whole gathered matrix (ring wrap-around)
  int Tm_p, Tn_p, n_ptm, n_ptn;     // producer tile and the number of tiles in the queue along rows / columns
  int rows_per_rank, rows_per_channel;
  int local_in_place;
  int k_chunks;                     // 1: one flag per channel.  > 1: n_ptn == k_chunks column tiles, one flag per (channel,
                                    // column tile) at flags[channel*k_chunks + tn], and the queue hands out column tile 0
                                    // of every row tile before column tile 1 (a consumer can start on the first K chunk)
  int interleave;                   // 0: the queue takes one source rank after the other.  1: the shard of first_src goes first
                                    // as a whole (the local one under the rotated orders); then row tile j of every other
                                    // rank comes before row tile j+1 of any, the order in which concurrent links deliver.
                                    // Needs at least two source ranks in the queue.
  unsigned pace_q8;                 // 0, or 256 x the ticks of the 100 MHz clock a link needs for one producer tile: a tile of
                                    // a remote shard is then not copied before its last byte would have arrived
  unsigned long long* pace_word;    // (epoch tag << 40 | start time) of the call in flight, set by its first producer
  unsigned epoch;
  unsigned wait_target;             // epoch * expected
  unsigned* flags;                  // [R*C*k_chunks]
  unsigned* ticket;                 // producer-tile queue head (grows by n_ptm*n_ptn per call)
  unsigned ticket_end;              // epoch * number of tickets per call (producer tiles + pushes)
  int n_out;                        // push mode: tickets n_ptm*n_ptn .. +n_out-1 each push one producer tile of the LOCAL shard
                                    // into one peer's copy of the gathered matrix (tile_push_data) and notify that peer
  bf16_t* peer_slots[kMaxWorld];    // where this rank's shard lands at peer q, [rows_per_rank, ld]; entry `rank` unused
  unsigned* pushed;                 // [R * channels per rank]: this rank's rows of channel c pushed into peer q at q*cpr + c
  WaitCtl ctl;
};

// ======================================================================================
// AllGather producer (pull mode).  Producer tiles form a queue that is consumed through an atomic
// ticket counter: ticket i is producer tile (tm, tn) in ring order over source ranks (by default
// rank+1, rank+2, ..., the local shard last).  Whoever holds a ticket copies that tile of the gathered
// matrix from its owner's shard and then notifies the tile's channel.  Dedicated producer
// workgroups drain the queue, and a GEMM workgroup whose channel is not ready yet takes tickets
// too instead of idling, so a consumer can never wait for a producer that is not resident.
// ======================================================================================
// Start time of the call in flight on the 100 MHz clock (low 40 bits), agreed on by all producers: the first one to
// find another call's tag in the word replaces it with this call's tag and its own clock reading.  One lane of wave 0
// of a workgroup tries the compare-and-swap (whichever workgroup's lands first wins); everybody then reads the word
// until it carries this call's tag.  Every branch is wave-uniform for the compiler too.
__device__ __forceinline__ unsigned long long pace_start(const AgProducer& p) {
  const unsigned long long mask40 = (1ull << 40) - 1, tag = (unsigned long long)(p.epoch & 0xffffffu) << 40;
  unsigned long long cur = uniform64(__hip_atomic_load(p.pace_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  if ((cur & ~mask40) != tag) {
    if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) == 0) lane0_cas64(p.pace_word, cur, tag | ((unsigned long long)wall_clock64() & mask40));
    // bounded: a caller that lets two calls share the workspace at the same time gets no pacing rather than a hang
    int tries = 0;
    do {
      cur = uniform64(__hip_atomic_load(p.pace_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    } while ((cur & ~mask40) != tag && ++tries < 4096);
    if ((cur & ~mask40) != tag) cur = 0;  // "started long ago": every tile is due
  }
  return cur & mask40;
}

// Called by every lane of one wave; the result is wave-uniform.
__device__ __forceinline__ bool claim_ticket(const AgProducer& p, unsigned* out) {
  const unsigned count = (unsigned)(p.n_ptm * p.n_ptn + p.n_out);
  unsigned t = lane0_fetch_add(p.ticket, 1u);
  unsigned idx = t - (p.ticket_end - count);
  // outside this call's range: the queue is empty (or the counter does not belong to this epoch, e.g. a workspace that
  // was not zeroed): give the ticket back; an index outside [0, count) is never handed out
  if (idx >= count) {
    lane0_add(p.ticket, 0xffffffffu);
    return false;
  }
  *out = idx;
  return true;
}

// All threads of the workgroup call this with the same ticket index; `wave` is the wave-uniform wave index.
// DEPTH = loads in flight per lane of the copy.
template <int DEPTH>
__device__ __forceinline__ void produce_tile(const AgProducer& p, int i, int tid, int wave, int nthreads) {
  const int ptm_per_rank = p.rows_per_rank / p.Tm_p;
  int tmi, tn;
  if (p.k_chunks > 1) { tn = i / p.n_ptm; tmi = i - tn * p.n_ptm; }
  else { tmi = i / p.n_ptn; tn = i - tmi * p.n_ptn; }
  int tm;
  if (p.interleave && tmi >= ptm_per_rank) {
    const int others = p.n_ptm / ptm_per_rank - 1;
    int r = tmi - ptm_per_rank, jm = r / others, s = r - jm * others;
    int q = p.first_src + 1 + s;
    if (q >= p.R) q -= p.R;
    tm = q * ptm_per_rank + jm;
  } else {
    tm = tmi + p.first_src * ptm_per_rank;  // ring order over source ranks: first_src, first_src+1, ...
    if (tm >= p.n_ptm_all) tm -= p.n_ptm_all;
  }
  int row_lo = tm * p.Tm_p;
  int src = tm / ptm_per_rank;                       // f_R
  int channel = tm / (p.rows_per_channel / p.Tm_p);  // f_C
  if (p.pace_q8 && src != p.rank) {
    // the links of all source ranks run side by side; this tile is number `nth` of what its rank sends
    const int jm = tm - src * ptm_per_rank;
    const int nth = p.k_chunks > 1 ? tn * ptm_per_rank + jm : jm * p.n_ptn + tn;
    const unsigned long long due = ((unsigned long long)(nth + 1) * p.pace_q8) >> 8;
    const unsigned long long t0 = pace_start(p);
    while ((((unsigned long long)wall_clock64() - t0) & ((1ull << 40) - 1)) < due) __builtin_amdgcn_s_sleep(8);
  }
  if (!(src == p.rank && p.local_in_place)) {
    const bf16_t* s = p.shards[src] + (long)(row_lo - src * p.rows_per_rank) * p.ld + (long)tn * p.Tn_p;
    bf16_t* d = p.gathered + (long)row_lo * p.ld + (long)tn * p.Tn_p;
    copy_tile<DEPTH>(s, p.ld, d, p.ld, p.Tm_p, p.Tn_p, tid, nthreads);
  }
  wait_all_vmem();  // this wave's written-through stores are complete ...
  __syncthreads();  // ... and so are every other wave's: the tile is where every die sees it
  if (wave == 0) lane0_add(p.flags + (p.k_chunks > 1 ? channel * p.k_chunks + tn : channel), 1u);
}

// Push mode (paper: "Data Primitives", push mode): ticket j of the push range is producer tile j % (tiles per shard) of the local shard,
// bound for peer rank+1+j/(tiles per shard).  The tile is written into that peer's copy of the gathered matrix and the
// peer's channel counter is raised (peer_tile_notify; here: the pushed counters).
template <int DEPTH>
__device__ __forceinline__ void push_tile(const AgProducer& p, int j, int tid, int wave, int nthreads) {
  const int tiles_per_shard = (p.rows_per_rank / p.Tm_p) * p.n_ptn;
  const int d = j / tiles_per_shard, t = j - d * tiles_per_shard;
  int q = p.rank + 1 + d;
  if (q >= p.R) q -= p.R;
  const int tm = t / p.n_ptn, tn = t - tm * p.n_ptn;
  const long off = (long)tm * p.Tm_p * p.ld + (long)tn * p.Tn_p;
  copy_tile<DEPTH>(p.shards[p.rank] + off, p.ld, p.peer_slots[q] + off, p.ld, p.Tm_p, p.Tn_p, tid, nthreads);
  wait_all_vmem();
  __syncthreads();  // every wave's written-through stores are complete
  const int cpr = p.rows_per_rank / p.rows_per_channel;
  if (wave == 0) lane0_add(p.pushed + q * cpr + (tm * p.Tm_p) / p.rows_per_channel, 1u);
}

// A claimed ticket of either kind.
template <int DEPTH>
__device__ __forceinline__ void work_ticket(const AgProducer& p, int i, int tid, int wave, int nthreads) {
  const int n_in = p.n_ptm * p.n_ptn;
  if (i < n_in) produce_tile<DEPTH>(p, i, tid, wave, nthreads);
  else push_tile<DEPTH>(p, i - n_in, tid, wave, nthreads);
}

// Every branch in the two loops below is wave-uniform for the compiler too (see lane0_fetch_add).
__device__ __forceinline__ void ag_producer(const AgProducer& p, int tid, int nthreads, int* s_ticket) {
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (;;) {
    if (wave == 0) {
      unsigned t;
      int v = claim_ticket(p, &t) ? (int)t : -1;
      *s_ticket = v;  // all lanes of wave 0 store the same value
    }
    __syncthreads();
    int i = __builtin_amdgcn_readfirstlane(*s_ticket);
    __syncthreads();
    if (i < 0) break;
    work_ticket<8>(p, i, tid, wave, nthreads);
  }
}

// consumer_tile_wait for the channels set in chan_mask (bit = global channel index; with K chunks: their first chunk) by a whole workgroup: while a channel is short of its target
// the workgroup works off producer tickets; with the queue empty it sleeps and polls (bounded by ctl.timeout).
// DEPTH = loads in flight per lane when this workgroup copies a producer tile itself: deep where the caller's registers allow
// (a ticket then takes a quarter of the time), shallow where they are full.
template <int DEPTH = 2>
__device__ __forceinline__ void consumer_wait_or_produce(const AgProducer& p, unsigned long long chan_mask, int tid, int nthreads, int* s_ticket) {
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned long long t0 = 0;
  if (wave == 0 && (p.ctl.timeout || p.pace_q8)) t0 = wall_clock64();
  // Tickets are taken only while the queue head has not passed the last tile of the awaited channels: beyond that point every
  // tile this workgroup needs is already in the hands of a resident workgroup, and taking more tickets would only delay it.
  int limit = 0;
  {
    const int tpc = p.rows_per_channel / p.Tm_p, ptm_per_rank = p.rows_per_rank / p.Tm_p;
    for (unsigned long long m = chan_mask; m; m &= m - 1) {
      int qi, qn;  // queue position (in row tiles) of the channel's first row tile, and of the one after its last
      const int ch0 = __builtin_ctzll(m), cpr = ptm_per_rank / tpc;
      if (p.interleave && ch0 / cpr != p.first_src) {
        const int others = p.n_ptm / ptm_per_rank - 1, c = ch0 % cpr;
        int s = ch0 / cpr - p.first_src - 1;
        if (s < 0) s += p.R;
        qi = ptm_per_rank + c * tpc * others + s;
        qn = ptm_per_rank + ((c + 1) * tpc - 1) * others + s + 1;
      } else {
        qi = __builtin_ctzll(m) * tpc - p.first_src * ptm_per_rank;
        if (qi < 0) qi += p.n_ptm_all;
        qn = qi + tpc;
      }
      int end = p.k_chunks > 1 ? qn : qn * p.n_ptn;  // with K chunks: the channel's tiles of chunk 0
      limit = end > limit ? end : limit;
    }
  }
  // With simulated links a ticket is a tile that may not be due for a long time: a consumer that took one would sleep on
  // it while its own rows arrive, and more workers do not make a link faster.  It only waits -- unless nothing has come
  // for far longer than a link takes (a millisecond): then no producer is running beside this kernel (a tool that runs
  // kernels one at a time, say), and the consumers work the queue off themselves as they do without links.
  const unsigned long long patience = p.pace_q8 ? 100000ull : 0ull;
  const unsigned queue_begin = p.ticket_end - (unsigned)(p.n_ptm * p.n_ptn + p.n_out);
  for (;;) {
    if (wave == 0) {
      int state = -2;  // -2: ready, -1: not ready and nothing to produce, >= 0: ticket to work off
      int first_short = 0;
      for (unsigned long long m = chan_mask; m; m &= m - 1) {
        int ch = __builtin_ctzll(m);
        unsigned f = __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.flags + ch * p.k_chunks, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        if ((int)(f - p.wait_target) < 0 && state == -2) { state = -1; first_short = ch; }
      }
      if (state == -1) {
        unsigned t;
        unsigned head = __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        if ((int)(head - queue_begin) < limit && (!patience || wall_clock64() - t0 > patience) && claim_ticket(p, &t)) state = (int)t;
        else if (p.ctl.timeout) {
          int st = __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.ctl.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
          if (st != 0) state = -2;  // abandoned elsewhere
          else if (wall_clock64() - t0 > p.ctl.timeout) {
            int expected = 0;  // every lane tries, the first one wins, all carry the same value
            __hip_atomic_compare_exchange_strong(p.ctl.status, &expected, 1 + first_short, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            state = -2;
          }
        }
      }
      *s_ticket = state;
    }
    __syncthreads();
    int state = __builtin_amdgcn_readfirstlane(*s_ticket);
    __syncthreads();
    if (state == -2) break;
    if (state >= 0) work_ticket<DEPTH>(p, state, tid, wave, nthreads);
    else __builtin_amdgcn_s_sleep(8);
  }
  acquire_after_wait(p.ctl);
  __syncthreads();
}


}  // namespace tl
