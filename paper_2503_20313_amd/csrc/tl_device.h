// Device-side building blocks shared by the fused kernels: signal primitives with
// acquire/release ordering (paper: "Signal Primitives", "Memory Consistency"), the
// schedule-position -> tile map, and coalesced tile copies ("Data Primitives").
// gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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
// die's caches before the producer wrote it.  The kernels here exclude that by construction:
//   * a kernel never reads a byte of flag-guarded data before it has seen the flag of the tile or
//     channel that byte belongs to (no prefetch across a wait, guarded regions are whole rows
//     aligned to more than a cache line), and
//   * lines cached by earlier kernels are dropped by the acquire every kernel dispatch performs.
// Hence every guarded line a die caches during a kernel was fetched after its producer's release.
// The default is therefore a workgroup-scope fence: it orders the workgroup's later loads after
// the flag load for the compiler and the wave, and leaves the caches alone.  Define
// TL_ACQ_SCOPE="agent" to build with the full device-scope acquire instead.
#ifndef TL_ACQ_SCOPE
#define TL_ACQ_SCOPE "workgroup"
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
};

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
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, TL_ACQ_SCOPE);
  return ok;
}

// ---------------------------------------------------------------------------------------
// Single-lane atomics without a divergent branch.  A loop whose body holds workgroup barriers
// must stay uniform for the compiler as well as at run time: with an `if (tid == 0)` around an
// atomic inside such a loop, the control-flow structurizer is free to rotate the divergent part
// across the loop's back edge, after which the waves of a workgroup no longer meet the same
// barrier in the same iteration.  These helpers are called by every lane of a wave; the atomic
// itself is issued for lane 0 only by narrowing EXEC inside one asm statement, and the result is
// returned as a wave-uniform value.  Device scope; ordering comes from the fences around them.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned lane0_fetch_add(unsigned* ptr, unsigned v) {
  unsigned r;
  unsigned long long saved;
  asm volatile(
      "s_mov_b64 %1, exec\n\t"
      "s_mov_b64 exec, 1\n\t"
      "global_atomic_add %0, %2, %3, off sc0\n\t"
      "s_waitcnt vmcnt(0)\n\t"
      "s_mov_b64 exec, %1"
      : "=&v"(r), "=&s"(saved)
      : "v"(ptr), "v"(v)
      : "memory");
  return __builtin_amdgcn_readfirstlane(r);
}

__device__ __forceinline__ void lane0_add(unsigned* ptr, unsigned v) {
  unsigned long long saved;
  asm volatile(
      "s_mov_b64 %0, exec\n\t"
      "s_mov_b64 exec, 1\n\t"
      "global_atomic_add %1, %2, off\n\t"
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
};

__host__ __device__ inline int sched_tile(const Sched& s, int p) {
  int l = p;
  if (s.swizzle && s.G % kXcds == 0) {
    int rnd = p / s.G, w = p - rnd * s.G;
    int span = s.n_tiles - rnd * s.G;
    if (span > s.G) span = s.G;
    if (span % kXcds == 0) l = rnd * s.G + (w % kXcds) * (span / kXcds) + w / kXcds;
  }
  int per_group = s.group_m * s.nbn;
  int g = l / per_group, within = l - g * per_group;
  int gsz = s.nbm - g * s.group_m;  // row blocks in this group (the last group may be short)
  if (gsz > s.group_m) gsz = s.group_m;
  int bn = within / gsz;
  int i = g * s.group_m + (within - bn * gsz);
  int bm = i + s.first_block;
  if (bm >= s.nbm) bm -= s.nbm;
  return bm * s.nbn + bn;
}

// ---------------------------------------------------------------------------------------
// Copy of a rows x cols (bf16, cols % 8 == 0) tile by one workgroup, 16 bytes per lane and
// access, four accesses in flight per lane.  Pointers must be 16-byte aligned and a tile must
// span less than 4 GiB in either matrix (offsets inside the tile are 32-bit, so that an access is
// a uniform base plus one offset register: the copy loops have to stay small enough in registers
// to share a SIMD with two waves of a matrix kernel).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void copy_tile(const bf16_t* __restrict__ src, long src_ld, bf16_t* __restrict__ dst, long dst_ld,
                                          int rows, int cols, int tid, int nthreads) {
  const int cpr = cols >> 3;  // 16-byte chunks per row
  const int total = rows * cpr;
  const int dr = nthreads / cpr, dc = nthreads - dr * cpr;  // chunk index + nthreads = (row + dr, chunk + dc) with carry
  const unsigned sld = (unsigned)src_ld * 2u, dld = (unsigned)dst_ld * 2u;
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
    for (int u = 0; u < 4; u++) *(u32x4*)(db + doff[u]) = v[u];
  }
  for (; i < total; i += nthreads) {
    *(u32x4*)(db + ((unsigned)r * dld + (unsigned)c * 16u)) =
        __builtin_nontemporal_load((const u32x4*)(sb + ((unsigned)r * sld + (unsigned)c * 16u)));
    r += dr; c += dc;
    if (c >= cpr) { c -= cpr; r++; }
  }
}

}  // namespace tl
