// Device-side building blocks shared by the fused kernels: signal primitives with
// acquire/release ordering (paper: "Signal Primitives", "Memory Consistency"), the
// schedule-position -> tile map, and coalesced tile copies ("Data Primitives").
// gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace tl {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Scope of the fence a consumer takes after it has seen a flag reach its target.
//
// The flag itself is always read with a device-scope atomic, and the producer's notify is a
// device-scope release (its data is written back to memory before the flag moves).  What the
// scope below decides is whether the consumer also discards the cached lines of its die: the
// eight dies have private L2s, so a device-scope acquire invalidates the whole L2 of the die and
// the L1 of the CU, and everything the other workgroups of that die were sharing there (weight
// panels, K/V blocks) has to be fetched again.  With one such acquire per tile wait this cost a
// tenth of the run time of the overlapped kernels.
//
// The invalidation guards against one thing only: a line of the awaited data that entered this
// die's caches before the producer wrote it.  The kernels here exclude that by construction when
//   * a kernel never reads a byte of flag-guarded data before it has seen the flag of the tile or
//     channel that byte belongs to (no prefetch across a wait),
//   * no cache line holds bytes of two differently guarded regions (else reading one region would
//     cache not-yet-written bytes of its neighbour): guarded regions start and end on 128-byte
//     boundaries.  Whole rows of the gathered matrices always do (their pitch is a multiple of 128
//     bytes); the column-split tiles of the ReduceScatter side do only for some shapes, so the host
//     decides per call and sets WaitCtl::strict where the condition fails, and
//   * lines cached by earlier kernels are dropped by the acquire every kernel dispatch performs.
// Then every guarded line a die caches during a kernel was fetched after its producer's release,
// and the fence after a wait only has to order the workgroup's later loads after the flag load for
// the compiler and the wave (workgroup scope), leaving the caches alone.  With WaitCtl::strict, or
// when built with TL_ACQ_SCOPE="agent", the full device-scope acquire is taken instead.
#ifndef TL_ACQ_SCOPE
#define TL_ACQ_SCOPE "workgroup"
#endif
#ifndef TL_COMPUTE_WAVE_PRIO
#define TL_COMPUTE_WAVE_PRIO 2
#endif
constexpr int kMaxWorld = 16;
constexpr int kXcds = 8;  // workgroup w of a launch runs on die w % 8

// ---------------------------------------------------------------------------------------
// Signal primitives.  A barrier is a counter that only grows; notify adds 1 with release
// ordering at device scope, wait spins until the counter reaches its target and then takes the
// acquire fence of scope TL_ACQ_SCOPE (see above), so that no later load of the waiting workgroup
// is issued before the flag was seen.  One lane per workgroup performs them; the caller brackets
// them with workgroup barriers.
// ---------------------------------------------------------------------------------------
struct WaitCtl {
  int* status;                 // status word: 0 = ok, else 1 + index of the flag whose wait expired
  unsigned long long timeout;  // in ticks of the 100 MHz wall clock; 0 = unbounded
  int strict;                  // 1: device-scope acquire after every wait (guarded regions share cache lines)
};

__device__ __forceinline__ void acquire_after_wait(const WaitCtl& ctl) {
  if (ctl.strict) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  else __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, TL_ACQ_SCOPE);
}

__device__ __forceinline__ void tile_notify(unsigned* flag, unsigned inc = 1u) {
  __hip_atomic_fetch_add(flag, inc, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// Returns false if the wait was abandoned (timeout here or earlier anywhere in the grid).
__device__ __forceinline__ bool tile_wait(const unsigned* flag, unsigned target, const WaitCtl& ctl, int flag_index) {
  unsigned long long t0 = 0;
  bool timed = ctl.timeout != 0;
  if (timed) t0 = wall_clock64();
  bool ok = true;
  while ((int)(__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
    __builtin_amdgcn_s_sleep(4);
    if (timed) {
      if (__hip_atomic_load(ctl.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { ok = false; break; }
      if (wall_clock64() - t0 > ctl.timeout) {
        int expected = 0;
        __hip_atomic_compare_exchange_strong(ctl.status, &expected, 1 + flag_index, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
        ok = false;
        break;
      }
    }
  }
  acquire_after_wait(ctl);
  return ok;
}

// tile_wait by all lanes of one wave, with every branch uniform for the compiler too (the polled values go through
// readfirstlane): for waits inside loops that hold workgroup barriers.  No acquire: the caller fences after the
// barrier that publishes the wait to the other waves.
__device__ __forceinline__ void wave_tile_wait(const unsigned* flag, unsigned target, const WaitCtl& ctl, int flag_index) {
  unsigned long long t0 = 0;
  const bool timed = ctl.timeout != 0;
  if (timed) t0 = wall_clock64();
  for (;;) {
    unsigned f = __builtin_amdgcn_readfirstlane(__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    if ((int)(f - target) >= 0) break;
    __builtin_amdgcn_s_sleep(4);
    if (timed) {
      int st = __builtin_amdgcn_readfirstlane(__hip_atomic_load(ctl.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
      if (st != 0) break;  // abandoned elsewhere
      if (wall_clock64() - t0 > ctl.timeout) {
        int expected = 0;  // every lane tries, the first one wins, all carry the same value
        __hip_atomic_compare_exchange_strong(ctl.status, &expected, 1 + flag_index, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
    }
  }
}

// 16-byte global store written through to device scope (sc1): once the wave's memory counter says it is complete it is
// visible to every die, so a producer that stores its tile this way can notify after a plain wait for its own stores,
// without the L2 write-back a release fence at device scope performs.
__device__ __forceinline__ void store16_device_scope(void* p, u32x4 v) {
  // the wait states behind it: a vector instruction may not overwrite the data registers of a store of more than 8 bytes
  // right after it, and the compiler does not look inside this statement
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
// ... with the address as a scalar base (the same for every lane) plus a 32-bit lane offset
__device__ __forceinline__ void store16_device_scope(const void* base, unsigned lane_off, u32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, %2 sc1\n\ts_nop 1" ::"v"(lane_off), "v"(v), "s"(base) : "memory");
}

// ---------------------------------------------------------------------------------------
// Clock sample of a launch: the first compute workgroup reads the shader-clock cycle counter and the 100 MHz wall clock
// when it starts and when it has finished its last tile, and leaves both differences in bytes 32..47 of the workspace
// (cycles, ticks): cycles / ticks x 100 = the shader clock in MHz the launch ran at, which on this chip depends on the
// operand data (measurement, read with tl_read_clocks).
// ---------------------------------------------------------------------------------------
struct ClockSample { long long cycles; unsigned long long ticks; };
__device__ __forceinline__ ClockSample clock_sample_begin(int compute_wg) {
  ClockSample c = {0, 0};
  if (compute_wg == 0) { c.cycles = clock64(); c.ticks = wall_clock64(); }
  return c;
}
__device__ __forceinline__ void clock_sample_end(const ClockSample& c0, int compute_wg, int* status_word) {
  if (compute_wg == 0 && threadIdx.x == 0) {
    long long* o = (long long*)status_word + 4;
    o[0] = clock64() - c0.cycles;
    o[1] = (long long)(wall_clock64() - c0.ticks);
  }
}

// ---------------------------------------------------------------------------------------
// Single-lane atomics without a divergent branch.  A loop whose body holds workgroup barriers
// must stay uniform for the compiler as well as at run time: with an `if (tid == 0)` around an
// atomic inside such a loop, the control-flow structurizer is free to rotate the divergent part
// across the loop's back edge, after which the waves of a workgroup no longer meet the same
// barrier in the same iteration.  These helpers are called by every lane of a wave; the atomic
// itself is issued for lane 0 only by narrowing EXEC inside one asm statement, and the result is
// returned as a wave-uniform value.  Device scope (sc1: performed where all eight dies see it, as the compiler
// does for an agent-scope atomic); ordering comes from the fences around them.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned lane0_fetch_add(unsigned* ptr, unsigned v) {
  unsigned r;
  unsigned long long saved;
  asm volatile(
      "s_mov_b64 %1, exec\n\t"
      "s_mov_b64 exec, 1\n\t"
      "global_atomic_add %0, %2, %3, off sc0 sc1\n\t"
      "s_waitcnt vmcnt(0)\n\t"
      "s_mov_b64 exec, %1"
      : "=&v"(r), "=&s"(saved)
      : "v"(ptr), "v"(v)
      : "memory");
  return __builtin_amdgcn_readfirstlane(r);
}

// 64-bit compare-and-swap by lane 0, no result: *ptr = desired if *ptr == expected.  Complete when it returns.
__device__ __forceinline__ void lane0_cas64(unsigned long long* ptr, unsigned long long expected, unsigned long long desired) {
  typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));
  const u64x2 data = {desired, expected};  // the instruction takes the new value in the low half, the comparand in the high half
  unsigned long long saved;
  asm volatile(
      "s_mov_b64 %0, exec\n\t"
      "s_mov_b64 exec, 1\n\t"
      "global_atomic_cmpswap_x2 %1, %2, off sc1\n\t"
      "s_waitcnt vmcnt(0)\n\t"
      "s_mov_b64 exec, %0"
      : "=&s"(saved)
      : "v"(ptr), "v"(data)
      : "memory");
}

__device__ __forceinline__ void lane0_add(unsigned* ptr, unsigned v) {
  unsigned long long saved;
  asm volatile(
      "s_mov_b64 %0, exec\n\t"
      "s_mov_b64 exec, 1\n\t"
      "global_atomic_add %1, %2, off sc1\n\t"
      "s_mov_b64 exec, %0"
      : "=&s"(saved)
      : "v"(ptr), "v"(v)
      : "memory");
}

// notify by a whole wave (uniform): release fence, then one add.
__device__ __forceinline__ void wave_tile_notify(unsigned* flag, unsigned inc = 1u) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  lane0_add(flag, inc);
}

// The tile movers below store written-through to device scope (sc1), so their data is where every die sees it as soon
// as the storing wave's memory counter says the stores are complete: a mover's notification is then
//   every wave: wait_all_vmem();  workgroup barrier;  one wave or lane: a relaxed add on the flag
// with no release fence, i.e. without the write-back of the die's L2 that such a fence performs (and waits for).
__device__ __forceinline__ void wait_all_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void notify_relaxed(unsigned* flag, unsigned inc = 1u) {
  __hip_atomic_fetch_add(flag, inc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A 64-bit value every lane holds alike, as a wave-uniform value for the compiler too.
__device__ __forceinline__ unsigned long long uniform64(unsigned long long v) {
  // the builtin returns int: through unsigned first, or a low word with its top bit set would sign-extend over the high word
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((unsigned)v), hi = (unsigned)__builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (unsigned long long)lo | ((unsigned long long)hi << 32);
}

// ---------------------------------------------------------------------------------------
// Tile order.  Position p of the schedule is computed by persistent workgroup p % G in its
// round p / G.  Inside a full round the workgroups of one die get a contiguous run of G/8
// logical tiles.  Logical tiles walk groups of `group_m` row blocks: inside a group the column
// block advances slowest and the row block fastest, so a run of consecutive logical tiles covers
// a compact (group_m x few columns) patch whose A rows and B columns are shared in the die's L2.
// Row blocks are optionally rotated so that `first_block` comes first.
// ---------------------------------------------------------------------------------------
struct Sched {
  int nbm, nbn, n_tiles, G;
  int first_block;  // rotation of row blocks (0 = natural)
  int swizzle;
  int group_m;      // >= 1
  int arrival_bpr = 0;  // 0, or the row blocks per rank: after the bpr blocks from first_block on (the local shard's), block j
                    // of each further rank along the ring comes before block j+1 of any
  int busy_first = 0;   // round 0: the workgroups that also have a tile in the partial last round take the first logical tiles
};

// Die swizzle alone: the logical index of schedule position p.
__host__ __device__ inline int sched_logical(const Sched& s, int p) {
  int l = p;
  if (s.swizzle && s.G % kXcds == 0) {
    int rnd = p / s.G, w = p - rnd * s.G;
    if (s.busy_first && rnd == 0 && s.n_tiles > s.G) {
      // A consumer whose first tiles wait for data that arrives in logical order: the workgroups w < tail run one tile
      // more than the others, so they get the earliest tiles [0, tail) and the others [tail, G), a run per die each.
      const int tail = s.n_tiles % s.G;
      if (tail && tail % kXcds == 0) {
        const int die = w % kXcds, i = w / kXcds, tb = tail / kXcds;
        return i < tb ? die * tb + i : tail + die * ((s.G - tail) / kXcds) + (i - tb);
      }
    }
    int span = s.n_tiles - rnd * s.G;
    if (span > s.G) span = s.G;
    if (span % kXcds == 0) l = rnd * s.G + (w % kXcds) * (span / kXcds) + w / kXcds;
  }
  return l;
}

// The other walk, for stages whose consumer needs a column block of EVERY row block before it can start (MoE part 2):
// groups of gb column blocks slowest, inside a group the row block next and the column block fastest.  gb = 1 finishes
// one column block of all rows at a time, but then all workgroups of the chip touch the same 512-byte slice of every
// row at once, and with a power-of-two row pitch those slices sit on a handful of memory channels; a few column
// blocks side by side spread the traffic while the consumer still gets complete columns early.
__host__ __device__ inline void colgroup_tile(int l, int nbm, int nbn, int gb, int* bm, int* bn) {
  int g = l / (nbm * gb), within = l - g * (nbm * gb);
  int gsz = nbn - g * gb;  // the last group may be narrower
  if (gsz > gb) gsz = gb;
  *bm = within / gsz;
  *bn = g * gb + (within - *bm * gsz);
}

__host__ __device__ inline int sched_tile(const Sched& s, int p) {
  int l = sched_logical(s, p);
  int per_group = s.group_m * s.nbn;
  int g = l / per_group, within = l - g * per_group;
  int gsz = s.nbm - g * s.group_m;  // row blocks in this group (the last group may be short)
  if (gsz > s.group_m) gsz = s.group_m;
  int bn = within / gsz;
  int i = g * s.group_m + (within - bn * gsz);
  int bm;
  if (s.arrival_bpr && i >= s.arrival_bpr) {
    const int others = s.nbm / s.arrival_bpr - 1;
    int r = i - s.arrival_bpr, j = r / others, q = r - j * others;
    bm = s.first_block + (q + 1) * s.arrival_bpr + j;
  } else {
    bm = i + s.first_block;
  }
  if (bm >= s.nbm) bm -= s.nbm;
  return bm * s.nbn + bn;
}

// ---------------------------------------------------------------------------------------
// Tile movers of the communication side: copy_tile (tile_push_data / tile_pull_data / rank_copy_data)
// and sum_tile (reduction of several source tiles).  A tile is rows x cols bf16 with cols % 8 == 0,
// 16-byte aligned, and spans less than 2 GiB in every matrix it lives in.
//
// These loops run beside two waves of a matrix kernel on every SIMD, which leaves them 48 vector
// registers, and a copy is bound by the bytes it keeps in flight: so all accesses of a lane use
// buffer addressing -- one resource descriptor per matrix in scalar registers, ONE lane-offset
// register, and a scalar offset that moves from step to step -- and eight 16-byte loads per lane
// are in flight at a time.  A "step" is one pass of the workgroup over nthreads consecutive
// 16-byte chunks; the tile shapes in use make a step either a block of whole rows (chunks per row
// divides nthreads) or a piece of one row (nthreads divides chunks per row), and in both cases a
// lane's chunk in step s is its chunk in step 0 shifted by a lane-independent offset.  Other shapes
// fall back to per-lane index arithmetic with four loads in flight.  The hardware range-checks a
// buffer access against the extent of the tile, so a wrong offset can return zeros but cannot fault.
// ---------------------------------------------------------------------------------------
typedef __amdgpu_buffer_rsrc_t rsrc_t;
// Cache policy of the movers' stores: sc1, written through to device scope.  Every tile a mover writes is followed by a
// device-scope release, which writes the die's dirty L2 lines back; lines that went through at once leave it less to
// do (measured: AllGather producer alone 0.075 -> 0.071 ms, K/V producer 0.360 -> 0.343 ms, MoE reduce side 0.129 ->
// 0.124 ms).  The same policy on the matrix kernels' epilogue stores costs them 4 %: those stay write-back.
#ifndef TL_SIDE_STORE_AUX
#define TL_SIDE_STORE_AUX 16
#endif

__device__ __forceinline__ rsrc_t tile_rsrc(const void* base, long ld, int rows, int cols) {
  unsigned bytes = (unsigned)(((long)(rows - 1) * ld + cols) * 2);
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

// Walk of the steps of a tile: for step s, off(ld_bytes) is the lane-independent byte offset of the step.
struct TileSteps {
  bool rows_mode;   // a step is dr whole rows; else a row takes spr steps
  int dr, spr, n_full, n_steps, nthreads;
  int lane_r, lane_c;  // the lane's chunk in step 0
  bool ok;
  __device__ __forceinline__ unsigned off(int s, unsigned ld_bytes) const {
    if (rows_mode) return (unsigned)(s * dr) * ld_bytes;
    int row = s / spr, sub = s - row * spr;
    return (unsigned)row * ld_bytes + (unsigned)(sub * nthreads) * 16u;
  }
};

__device__ __forceinline__ TileSteps tile_steps(int rows, int cpr, int tid, int nthreads) {
  TileSteps t;
  t.nthreads = nthreads;
  t.ok = true;
  t.rows_mode = cpr <= nthreads;
  if (t.rows_mode) {
    t.dr = nthreads / cpr; t.spr = 1;
    t.ok = t.dr * cpr == nthreads;
    t.lane_r = tid / cpr; t.lane_c = tid - t.lane_r * cpr;
    t.n_full = rows / t.dr; t.n_steps = (rows + t.dr - 1) / t.dr;
  } else {
    t.dr = 0; t.spr = cpr / nthreads;
    t.ok = t.spr * nthreads == cpr;
    t.lane_r = 0; t.lane_c = tid;
    t.n_full = t.n_steps = rows * t.spr;
  }
  return t;
}

__device__ __forceinline__ u32x4 buf_load16(rsrc_t r, unsigned lane_off, unsigned step_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)step_off, 2 /* streaming */);
}
__device__ __forceinline__ void buf_store16(u32x4 v, rsrc_t r, unsigned lane_off, unsigned step_off) {
  __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)lane_off, (int)step_off, TL_SIDE_STORE_AUX);
}

template <int DEPTH = 8>  // loads in flight per lane
__device__ __forceinline__ void copy_tile(const bf16_t* __restrict__ src, long src_ld, bf16_t* __restrict__ dst, long dst_ld,
                                          int rows, int cols, int tid, int nthreads) {
  const int cpr = cols >> 3;  // 16-byte chunks per row
  const unsigned sld = (unsigned)src_ld * 2u, dld = (unsigned)dst_ld * 2u;
  const TileSteps ts = tile_steps(rows, cpr, tid, nthreads);
  if (ts.ok) {
    const rsrc_t rs = tile_rsrc(src, src_ld, rows, cols), rd = tile_rsrc(dst, dst_ld, rows, cols);
    const unsigned so = (unsigned)ts.lane_r * sld + (unsigned)ts.lane_c * 16u, dof = (unsigned)ts.lane_r * dld + (unsigned)ts.lane_c * 16u;
    int st = 0;
    for (; st + DEPTH <= ts.n_full; st += DEPTH) {
      u32x4 v[DEPTH];
#pragma unroll
      for (int u = 0; u < DEPTH; u++) v[u] = buf_load16(rs, so, ts.off(st + u, sld));
#pragma unroll
      for (int u = 0; u < DEPTH; u++) buf_store16(v[u], rd, dof, ts.off(st + u, dld));
    }
    for (; st + 2 <= ts.n_full; st += 2) {
      u32x4 v0 = buf_load16(rs, so, ts.off(st, sld)), v1 = buf_load16(rs, so, ts.off(st + 1, sld));
      buf_store16(v0, rd, dof, ts.off(st, dld));
      buf_store16(v1, rd, dof, ts.off(st + 1, dld));
    }
    for (; st < ts.n_steps; st++)   // at most one full step, then the partial one (rows mode): predicated per lane
      if (st < ts.n_full || st * ts.dr + ts.lane_r < rows) buf_store16(buf_load16(rs, so, ts.off(st, sld)), rd, dof, ts.off(st, dld));
    return;
  }
  const int total = rows * cpr;
  const int dr = nthreads / cpr, dc = nthreads - dr * cpr;  // chunk index + nthreads = (row + dr, chunk + dc) with carry
  const char* sb = (const char*)src;
  char* db = (char*)dst;
  int r = tid / cpr, c = tid - r * cpr;
  int i = tid;
  for (; i + 3 * nthreads < total; i += 4 * nthreads) {
    u32x4 v[4];
    unsigned doff[4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
      v[u] = __builtin_nontemporal_load((const u32x4*)(sb + ((unsigned)r * sld + (unsigned)c * 16u)));
      doff[u] = (unsigned)r * dld + (unsigned)c * 16u;
      r += dr; c += dc;
      if (c >= cpr) { c -= cpr; r++; }
    }
#pragma unroll
    for (int u = 0; u < 4; u++) store16_device_scope(db + doff[u], v[u]);
  }
  for (; i < total; i += nthreads) {
    store16_device_scope(db + ((unsigned)r * dld + (unsigned)c * 16u),
                         __builtin_nontemporal_load((const u32x4*)(sb + ((unsigned)r * sld + (unsigned)c * 16u))));
    r += dr; c += dc;
    if (c >= cpr) { c -= cpr; r++; }
  }
}

// dst tile = bf16( sum over n_src source tiles, fp32, in source order ).  src(q) returns the uniform base pointer of
// source q's tile; all sources share the row pitch src_ld.  Up to DEPTH sources of one chunk are in flight.
__device__ __forceinline__ void acc_bf16x8(float (&s)[8], u32x4 v) {
#pragma unroll
  for (int e = 0; e < 4; e++) {
    s[2 * e] += __uint_as_float(v[e] << 16);
    s[2 * e + 1] += __uint_as_float(v[e] & 0xffff0000u);
  }
}

__device__ __forceinline__ u32x4 pack_bf16x8(const float (&s)[8]) {
  bf16x8 v;
#pragma unroll
  for (int e = 0; e < 8; e++) v[e] = (bf16_t)s[e];
  return __builtin_bit_cast(u32x4, v);
}

template <int DEPTH = 4, int POS = 1, class SrcFn>  // DEPTH sources of POS chunks in flight per lane
__device__ __forceinline__ void sum_tile(SrcFn src, int n_src, bf16_t* dst, long src_ld, long dst_ld, int rows, int cols, int tid,
                                         int nthreads) {
  const int cpr = cols >> 3;
  const unsigned sld = (unsigned)src_ld * 2u, dld = (unsigned)dst_ld * 2u;
  const TileSteps ts = tile_steps(rows, cpr, tid, nthreads);
  if (ts.ok) {
    const rsrc_t rd = tile_rsrc(dst, dst_ld, rows, cols);
    const unsigned so = (unsigned)ts.lane_r * sld + (unsigned)ts.lane_c * 16u, dof = (unsigned)ts.lane_r * dld + (unsigned)ts.lane_c * 16u;
    // NP chunks (steps st .. st+NP-1) of this lane: sum their sources, store
    auto group = [&](auto np_c, int st) {
      constexpr int NP = decltype(np_c)::value;
      float s[NP][8];
#pragma unroll
      for (int w = 0; w < NP; w++)
#pragma unroll
        for (int e = 0; e < 8; e++) s[w][e] = 0.f;
      for (int q0 = 0; q0 < n_src; q0 += DEPTH) {
        u32x4 v[NP][DEPTH];
#pragma unroll
        for (int u = 0; u < DEPTH; u++)
          if (q0 + u < n_src) {  // uniform condition
            const rsrc_t rq = tile_rsrc(src(q0 + u), src_ld, rows, cols);
#pragma unroll
            for (int w = 0; w < NP; w++) v[w][u] = buf_load16(rq, so, ts.off(st + w, sld));
          }
#pragma unroll
        for (int u = 0; u < DEPTH; u++)
          if (q0 + u < n_src) {
#pragma unroll
            for (int w = 0; w < NP; w++) acc_bf16x8(s[w], v[w][u]);
          }
      }
#pragma unroll
      for (int w = 0; w < NP; w++) buf_store16(pack_bf16x8(s[w]), rd, dof, ts.off(st + w, dld));
    };
    int st = 0;
    if (n_src == 2) {
      // two sources (top-2 routing): no running sums to keep, so the registers hold eight loads in flight instead
      // (four chunks of both sources); a chunk's sum lives only between its unpacking and its store
      const rsrc_t r0 = tile_rsrc(src(0), src_ld, rows, cols), r1 = tile_rsrc(src(1), src_ld, rows, cols);
      for (; st + 4 <= ts.n_full; st += 4) {
        u32x4 a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
          a[u] = buf_load16(r0, so, ts.off(st + u, sld));
          b[u] = buf_load16(r1, so, ts.off(st + u, sld));
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
          float s[8];
#pragma unroll
          for (int e = 0; e < 4; e++) {
            s[2 * e] = __uint_as_float(a[u][e] << 16) + __uint_as_float(b[u][e] << 16);
            s[2 * e + 1] = __uint_as_float(a[u][e] & 0xffff0000u) + __uint_as_float(b[u][e] & 0xffff0000u);
          }
          buf_store16(pack_bf16x8(s), rd, dof, ts.off(st + u, dld));
        }
      }
    }
    for (; st + POS <= ts.n_full; st += POS) group(std::integral_constant<int, POS>{}, st);
    for (; st < ts.n_steps; st++)   // fewer than POS full steps, then the partial one (rows mode): predicated per lane
      if (st < ts.n_full || st * ts.dr + ts.lane_r < rows) group(std::integral_constant<int, 1>{}, st);
    return;
  }
  const int total = rows * cpr;
  const int dr = nthreads / cpr, dc = nthreads - dr * cpr;
  char* db = (char*)dst;
  int r = tid / cpr, c = tid - r * cpr;
  for (int i = tid; i < total; i += nthreads) {
    const unsigned so = (unsigned)r * sld + (unsigned)c * 16u;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int q = 0; q < n_src; q++) acc_bf16x8(s, __builtin_nontemporal_load((const u32x4*)((const char*)src(q) + so)));
    store16_device_scope(db + ((unsigned)r * dld + (unsigned)c * 16u), pack_bf16x8(s));
    r += dr; c += dc;
    if (c >= cpr) { c -= cpr; r++; }
  }
}

}  // namespace tl
