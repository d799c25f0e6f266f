// One bf16 GEMM output tile on CDNA4 matrix cores: C[BM,BN] = A[BM,K] . B[K,BN], A row-major
// (K contiguous), B row-major as [K,N] (N contiguous), fp32 accumulation, bf16 (RNE) output.
//
// Design (gfx950):
//  * global -> LDS with 16-byte direct-to-LDS loads (no register staging) into a ring of NS
//    stages of BK k-values each.  The loads of a stage are requested NS-1 steps before they are
//    used, so that several stages are in flight per compute unit at any time: measured on
//    MI355X, a single stage in flight leaves the kernel bound by the latency of the load path.
//    The bijection between 16-byte chunks and LDS slots is chosen so that the later fragment
//    reads are bank-conflict free (A: chunk index XOR a function of the row; B with a
//    power-of-two row pitch: 64-byte group XOR k%4; B tiles 224 wide need none).
//  * the MFMA "A" operand is taken from the B tile with transposing LDS reads
//    (ds_read_b64_tr_b16: a 16-lane block reads 4 k-rows x 16 columns and hands each lane the
//    4 k-values of its column), the MFMA "B" operand from the A tile with 16-byte reads; the
//    product is therefore the transposed tile C^T, whose accumulator layout gives every lane
//    4 consecutive columns of one row of C; the epilogue passes them through LDS to store whole lines.
//  * v_mfma_f32_32x32x16_bf16, wave tile (BM/WM) x (BN/WN).
#pragma once
#include <type_traits>

#include "tl_device.h"

namespace tl {

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

template <int BM_, int BN_, int WM_, int WN_, int BK_ = 32, int NS_ = 4>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, NS = NS_, WM = WM_, WN = WN_;
  static constexpr int NWAVES = WM * WN, NTHREADS = NWAVES * 64;
  static constexpr int WTM = BM / WM, WTN = BN / WN, MT = WTM / 32, NT = WTN / 32;
  static constexpr int SL = BK / 16;              // 16-wide k-slices (one MFMA deep) per stage
  static constexpr int A_CPR = BK / 8;            // 16-byte chunks per row of the A tile
  static constexpr int A_RPB = 256 / (BK * 2);    // A rows per 256 bytes of LDS (all 64 banks)
  static constexpr int A_PITCH = BK * 2;          // bytes per A row in LDS
  static constexpr int A_LOADS = BM * A_CPR / 64; // wave-wide 1 KiB loads per stage, A tile
  static constexpr int B_CPR = BN / 8;            // 16-byte chunks per k-row of the B tile
  static constexpr int B_LOADS = BK * B_CPR / 64;
  static constexpr bool B_SWZ = (B_CPR % 16) == 0;
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BK * BN * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  // Epilogue staging: every wave passes its WTM x WTN result through an LDS region of its own, rows padded by 16 bytes.
  static constexpr int EP_PITCH = WTN * 2 + 16;
  static constexpr int EP_BYTES = NWAVES * WTM * EP_PITCH;
  static constexpr int LDS_BYTES = NS * STAGE_BYTES > EP_BYTES ? NS * STAGE_BYTES : EP_BYTES;
  static_assert((WTM * (WTN / 8)) % 64 == 0, "the epilogue hands out 16-byte chunks of the wave tile 64 at a time");
  static constexpr int A_PER_WAVE = (A_LOADS + NWAVES - 1) / NWAVES;
  static constexpr int B_PER_WAVE = (B_LOADS + NWAVES - 1) / NWAVES;
  // Direct-to-LDS loads per stage issued by every wave.  Every wave issues the same number (the vmcnt
  // bookkeeping relies on it): where the loads do not divide evenly, the surplus waves repeat the last one.
  static constexpr int LPW = A_PER_WAVE + B_PER_WAVE;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  static_assert(SL % 2 == 0, "fragment double buffering assumes an even number of k-slices per stage");
  static_assert((NS - 1) * LPW <= 63, "vmcnt is a 6-bit counter");
};

// Sixteen zero bytes: what a lane loads in place of a piece of A or B beyond the end of K.
static __device__ __attribute__((aligned(16))) unsigned g_zero_chunk[4];

__device__ __forceinline__ void lds_load16(const void* g, char* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// The same load with the global address given as a scalar base (the same for every lane) plus a 32-bit lane offset:
// advancing the address from one K step to the next is then scalar arithmetic.  The compiler's builtin always takes the
// per-lane 64-bit form, hence the instruction is written out; M0 carries the wave's LDS destination (lane l lands at
// M0 + 16 l).  One wait state between the write of M0 and its use by the load.
__device__ __forceinline__ void lds_load16_sbase(const char* base, unsigned lane_off, unsigned lds_wave_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_wave_base), "v"(lane_off), "s"(base) : "memory");
}
// ... and with a per-lane 64-bit address, the LDS destination given as a 32-bit LDS address.
__device__ __forceinline__ void lds_load16_at(const char* g, unsigned lds_wave_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_wave_base), "v"(g) : "memory");
}

__device__ __forceinline__ short4_t lds_read_tr(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)p);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N <= 63, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Where the rows of an output tile go: dense = row r of the tile at c + r*ldc, unscaled.
struct DenseRows {
  static constexpr bool SCALED = false, GATED = false;
  bf16_t* c;
  long ldc;
  __device__ __forceinline__ bf16_t* row(int r, float& scale) const { return c + (long)r * ldc; }
  // 8 consecutive bf16 of tile row r starting at tile column col (col % 8 == 0)
  __device__ __forceinline__ void group(int /*r0*/) const {}
  __device__ __forceinline__ void store(int r, int col, u32x4 v) const { *(u32x4*)(c + (long)r * ldc + col) = v; }
};

// Hook of gemm_tile for A operands that arrive in chunks along K: before the loads of K step `ks` are requested,
// gemm_tile calls wait(ks) from every thread whenever starts(ks) holds, and acquire() after the barrier that follows.
// The steps of the pipeline's prologue (ks < NS) are not announced: they belong to what the caller waited for.
struct NoKWait {
  static constexpr bool ENABLED = false;
  __device__ __forceinline__ bool starts(int) const { return false; }
  __device__ __forceinline__ void wait(int) const {}
  __device__ __forceinline__ void acquire() const {}
};

// Hook of gemm_tile for work that has to wait until this workgroup's earlier global stores are complete (the deferred
// producer_tile_notify of the previous tile): when pending() holds, the prologue waits for ALL outstanding vector memory
// operations of every wave instead of for the first stage only -- the stores of the previous tile's epilogue were issued
// before this tile's loads and have long been on their way -- and run() is called by every thread right after the
// workgroup barrier that follows.
struct NoHook {
  __device__ __forceinline__ bool pending() const { return false; }
  __device__ __forceinline__ void run() const {}
};

// Output of a GEMM whose B holds a gate and an up projection side by side, 32 columns of the one, then the same 32
// features of the other (so that the two values of a feature sit in the same lane, in neighbouring 32x32 accumulator
// blocks): the tile stores act(gate) * up, half as many columns as it computes (the activation between the two halves
// of the MLP layer in the paper's evaluation, applied to the unrounded accumulators).  `c` points at the tile's first
// output column (half the tile's first GEMM column).
enum { ACT_SILU_MUL = 1, ACT_GELU_MUL = 2 };
struct GatedRows {
  static constexpr bool SCALED = false, GATED = true;
  bf16_t* c;
  long ldc;
  int act;
  __device__ __forceinline__ bf16_t* row(int r, float& scale) const { return c + (long)r * ldc; }
  __device__ __forceinline__ void group(int /*r0*/) const {}
  __device__ __forceinline__ void store(int r, int col, u32x4 v) const { *(u32x4*)(c + (long)r * ldc + col) = v; }
  __device__ __forceinline__ float apply(float g, float u) const {
    if (act == ACT_SILU_MUL) return g * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * u;  // g * sigmoid(g) * u
    return 0.5f * g * (1.f + erff(g * 0.70710678118654752f)) * u;                                                          // g * Phi(g) * u
  }
};

// Computes one output tile.  `a` points at column 0 of the A rows: tile row r is A row r, or A row
// a_rows[r] / a_div when a_rows is given (row gather: the tile's rows are picked by index; the picked rows must lie
// within 4 GiB of `a`); `b` points at row 0 of B at the tile's first column; both are the same for every lane.
// `out.row(r, scale)` gives the address of the tile's first
// column in output row r (and a per-row factor applied in fp32 before rounding if Out::SCALED);
// `out.store(r, col, v, r0)` stores 8 rounded values of row r (a functor may do more with them, e.g. reduce); r0 is the
// first of the consecutive rows that the same store instruction covers (no lane's row is below it), the same for every lane, so that a
// functor whose destination depends on the row can decide per instruction instead of per lane.  gemm_tile works on a copy
// of the functor, which may therefore keep state from one store to the next.
// With Out::GATED the tile's columns come in pairs of 32 (gate, up): out.apply(gate, up) is stored, at half the column.
// rows/cols = valid extent of the tile (ragged edges): loads are clamped to valid memory, stores are
// masked.  K % 8 == 0 (rows of A start on 16-byte boundaries); a last K step shorter than BK is filled up with zeros:
// the 16-byte pieces of it that lie beyond K are loaded from a block of zeros instead of from the matrices (every lane
// of a direct-to-LDS load names its own global address), so both operands of the surplus products are zero.
// All threads of the workgroup must call it; it ends with all LDS accesses complete.
//
// LDS: the NS stages of the A tile, then the NS stages of the B tile.  The K loop is unrolled NS times so that the ring
// slot of every stage is a compile-time constant: all fragment reads then address LDS as (a lane register fixed for the
// whole tile) + (an immediate), and the direct-to-LDS loads as (a scalar base that advances per K step) + (a lane
// offset fixed for the whole tile).  The loop body is left with no vector-ALU instruction besides the matrix ones:
// measured, every vector instruction taken out of this loop shortened it, in cycles and -- on a chip that runs the
// matrix cores at its power limit -- in clock.
template <class Cfg, class Out, class KW = NoKWait, class Hook = NoHook>
__device__ __forceinline__ void gemm_tile(const bf16_t* __restrict__ a, long lda, const int* __restrict__ a_rows, int a_div,
                                          const bf16_t* __restrict__ b, long ldb, const Out& out, int rows, int cols, int K,
                                          char* smem, const KW& kw = KW{}, const Hook& hook = Hook{}) {
  constexpr int NS = Cfg::NS, SL = Cfg::SL, LPW = Cfg::LPW;
  constexpr int A_REGION = NS * Cfg::A_BYTES;   // the B stages start here
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform for the compiler too
  const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;
  // ---- this wave's share of the stage loads: a scalar base per matrix and a lane offset per load
  unsigned a_voff[Cfg::A_PER_WAVE], b_voff[Cfg::B_PER_WAVE];
  K = __builtin_amdgcn_readfirstlane(K);   // the trip counts of the K loops must be uniform for the compiler too
  const int k_tail = K % Cfg::BK;  // k-values of the last K step if it is a short one, else 0
  unsigned tail_ok = 0;            // bit L: this lane's load L of the short step lies inside K
#pragma unroll
  for (int i = 0; i < Cfg::A_PER_WAVE; i++) {
    int j = wave + i * Cfg::NWAVES;  // wave-load index: LDS slots [64j, 64j+64)
    if (j >= Cfg::A_LOADS) j = Cfg::A_LOADS - 1;
    int slot = j * 64 + lane;
    int row = slot / Cfg::A_CPR;
    int chunk = (slot % Cfg::A_CPR) ^ ((row / Cfg::A_RPB) % Cfg::A_CPR);  // logical 16-byte chunk stored at this slot
    int grow = row < rows ? row : rows - 1;
    if (a_rows) grow = a_rows[grow] / a_div;
    a_voff[i] = (unsigned)grow * (unsigned)(lda * 2) + (unsigned)(chunk * 16);
    if (chunk * 8 < k_tail) tail_ok |= 1u << i;
  }
#pragma unroll
  for (int i = 0; i < Cfg::B_PER_WAVE; i++) {
    int j = wave + i * Cfg::NWAVES;
    if (j >= Cfg::B_LOADS) j = Cfg::B_LOADS - 1;
    int slot = j * 64 + lane;
    int k = slot / Cfg::B_CPR, ncp = slot - k * Cfg::B_CPR;
    int nc = Cfg::B_SWZ ? (ncp ^ ((k & 3) << 2)) : ncp;
    int col = nc * 8 < cols ? nc * 8 : cols - 8;
    b_voff[i] = (unsigned)k * (unsigned)(ldb * 2) + (unsigned)(col * 2);
    if (k < k_tail) tail_ok |= 1u << (Cfg::A_PER_WAVE + i);
  }
  // scalar registers hold the two bases; they advance by one K step per requested stage
  const char* a_base = (const char*)uniform64((unsigned long long)a);
  const char* b_base = (const char*)uniform64((unsigned long long)b);
  // (made uniform explicitly: inside a function that is not inlined the arguments arrive in vector registers)
  const long b_step = (long)uniform64((unsigned long long)(ldb * Cfg::BK * 2));  // bytes per K-step
  const unsigned smem_u = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)smem);

  // Load number L (0..LPW-1) of this wave's share of the stage the bases point at, into ring slot `slot`:
  // loads 0..A_PER_WAVE-1 belong to the A tile, the rest to the B tile.  `tail` (compile-time): the stage is the short
  // last K step, lanes whose piece lies beyond K load zeros.
  auto issue_load = [&](int slot, auto l_c, auto tail_c) {
    constexpr int L = decltype(l_c)::value;
    constexpr bool TAIL = decltype(tail_c)::value;
    constexpr bool IS_A = L < Cfg::A_PER_WAVE;
    constexpr int LL = IS_A ? L : L - Cfg::A_PER_WAVE;
    int j = wave + LL * Cfg::NWAVES;
    if (j >= (IS_A ? Cfg::A_LOADS : Cfg::B_LOADS)) j = (IS_A ? Cfg::A_LOADS : Cfg::B_LOADS) - 1;
    const unsigned lds = smem_u + (IS_A ? slot * Cfg::A_BYTES : A_REGION + slot * Cfg::B_BYTES) + j * 1024;
    unsigned voff;
    if constexpr (IS_A) voff = a_voff[LL]; else voff = b_voff[LL];
    const char* base = IS_A ? a_base : b_base;
    if constexpr (TAIL) {
      const char* src = ((tail_ok >> L) & 1u) ? base + voff : (const char*)g_zero_chunk;
      lds_load16_at(src, lds);
    } else {
      lds_load16_sbase(base, voff, lds);
    }
  };
  auto issue_stage = [&](int slot, auto tail_c) {
    static_for<0, LPW>([&](auto l_c) { issue_load(slot, l_c, tail_c); });
    a_base += Cfg::BK * 2;
    b_base += b_step;
  };

  // ---- per-lane LDS read addresses (fixed for the tile; the stage and slice offsets are immediates)
  // A fragment (MFMA B operand): lane holds row (lane%32) of the wave's m-tile, k = 8*(lane/32)..+7 of the 16-wide k-slice.
  const int a_row = wm * Cfg::WTM + (lane & 31);
  const int a_x = (lane >> 5) ^ ((a_row / Cfg::A_RPB) % Cfg::A_CPR);
  const char* a_rd[SL];
#pragma unroll
  for (int sl = 0; sl < SL; sl++) a_rd[sl] = smem + a_row * Cfg::A_PITCH + ((a_x ^ (2 * sl)) << 4);
  // B fragment (MFMA A operand) via transposing reads: lane supplies the address of k-row
  // 8*(lane/32) + (lane%16)/4 (+4 for the second read), columns 16*((lane/16)%2) + 4*(lane%4)..+3.
  const int b_k = 8 * (lane >> 5) + ((lane & 15) >> 2);
  const int b_n = wn * Cfg::WTN + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const char* b_rd[Cfg::NT];
#pragma unroll
  for (int nt = 0; nt < Cfg::NT; nt++) {
    int n = b_n + nt * 32;
    int nc = n >> 3;
    if (Cfg::B_SWZ) nc ^= (b_k & 3) << 2;
    b_rd[nt] = smem + A_REGION + (b_k * Cfg::B_CPR + nc) * 16 + (n & 4) * 2;
  }

  floatx16 acc[Cfg::MT][Cfg::NT];
#pragma unroll
  for (int mt = 0; mt < Cfg::MT; mt++)
#pragma unroll
    for (int nt = 0; nt < Cfg::NT; nt++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[mt][nt][e] = 0.f;

  bf16x8 af[2][Cfg::MT], bfr[2][Cfg::NT];
  // One LDS fragment read of k-slice `sl` of the stage in ring slot `slot` into register set BUF:
  // reads 0..NT-1 fetch the B fragments (two transposing reads each), NT..NT+MT-1 the A fragments.
  constexpr int N_READS = Cfg::NT + Cfg::MT;
  constexpr int N_MFMA = Cfg::MT * Cfg::NT;
  auto read_frag = [&](int slot, auto sl_c, auto buf_c, auto r_c) {
    constexpr int BUF = decltype(buf_c)::value, R = decltype(r_c)::value, S = decltype(sl_c)::value;
    if constexpr (R < Cfg::NT) {
      const char* p = b_rd[R] + slot * Cfg::B_BYTES + S * 16 * Cfg::B_CPR * 16;
      short4_t lo = lds_read_tr(p);
      short4_t hi = lds_read_tr(p + 4 * Cfg::B_CPR * 16);
      typedef short short8_t __attribute__((ext_vector_type(8)));
      short8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      bfr[BUF][R] = __builtin_bit_cast(bf16x8, v);
    } else {
      constexpr int MTI = R - Cfg::NT;
      af[BUF][MTI] = *(const bf16x8*)(a_rd[S] + slot * Cfg::A_BYTES + MTI * 32 * Cfg::A_PITCH);
    }
  };
  using std::integral_constant;
  typedef integral_constant<bool, true> yes;
  typedef integral_constant<bool, false> no;
  // One k-slice in fixed program order: the MFMAs of the slice held in register set CUR, with the
  // fragment reads of the following slice (k-slice RSL of the stage in ring slot rslot) placed after the first
  // MFMA, RPG per MFMA: no read sits between the wait for this slice's fragments and its first MFMA,
  // and the last read still has several MFMAs of cover.  BS = position of the slice in the loop body
  // (which spans SL slices; -1 = outside the loop): with ISSUE, the LPW global loads of a newly requested stage (ring
  // slot islot) are spread evenly over the body's MFMAs, one at a time, so that no wave sits in a full
  // memory-instruction queue while its MFMAs wait behind it.
  auto slice = [&](auto cur_c, auto bs_c, auto reads_c, int rslot, auto rsl_c, auto issue_c, auto tail_c, int islot) {
    constexpr int CUR = decltype(cur_c)::value, BS = decltype(bs_c)::value;
    constexpr bool READS = decltype(reads_c)::value, ISSUE = decltype(issue_c)::value;
    constexpr int GAPS = N_MFMA > 2 ? N_MFMA - 2 : 1;
    constexpr int RPG = (N_READS + GAPS - 1) / GAPS;
    static_for<0, N_MFMA>([&](auto m_c) {
      constexpr int M = decltype(m_c)::value;
      constexpr int MTI = M / Cfg::NT, NTI = M % Cfg::NT;
      acc[MTI][NTI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[CUR][NTI], af[CUR][MTI], acc[MTI][NTI], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (BS >= 0 && ISSUE) {
        constexpr int G = BS * N_MFMA + M;  // MFMA index inside the loop body
        static_for<0, LPW>([&](auto l_c) {
          constexpr int L = decltype(l_c)::value;
          if constexpr (G == ((2 * L + 1) * SL * N_MFMA) / (2 * LPW)) {
            issue_load(islot, l_c, tail_c);
            __builtin_amdgcn_sched_barrier(0);
          }
        });
      }
      if constexpr (READS) {
        static_for<M * RPG, ((M + 1) * RPG < N_READS ? (M + 1) * RPG : N_READS)>([&](auto r_c) {
          read_frag(rslot, rsl_c, integral_constant<int, CUR ^ 1>{}, r_c);
        });
        __builtin_amdgcn_sched_barrier(0);
      }
    });
  };

  // K loop: BK per step, ring of NS LDS stages, stage s lives in slot s % NS.  A loop body starts at
  // the barrier:
  //   wait + barrier : stage s+1 has landed for every wave; nobody reads stage s from LDS any more
  //                    (the fragments of its last slice are already in registers)
  //   body slice 0   : multiply the last slice of stage s, read (stage s+1, slice 0)
  //   body slice j>0 : multiply slice j-1 of stage s+1, read (stage s+1, slice j)
  //   throughout     : request stage s+NS into the slot stage s just left, one load at a time
  // The last NS bodies request nothing and wait for all outstanding loads instead; the body that requests a short
  // last stage is a copy of its own.
  const int nk = (K + Cfg::BK - 1) / Cfg::BK;
  static_for<0, NS>([&](auto s_c) {
    constexpr int S = decltype(s_c)::value;
    if (S < nk) {
      if (k_tail != 0 && S == nk - 1) issue_stage(S, yes{}); else issue_stage(S, no{});
    }
  });
  const bool hooked = hook.pending();
  if (nk >= NS && !hooked) wait_vmcnt<(NS - 1) * LPW>(); else wait_vmcnt<0>();
  __syncthreads();
  if (hooked) hook.run();
  static_for<0, N_READS>([&](auto r_c) { read_frag(0, integral_constant<int, 0>{}, integral_constant<int, 0>{}, r_c); });
  static_for<0, SL - 1>([&](auto sl_c) {
    constexpr int S = decltype(sl_c)::value;
    slice(integral_constant<int, S & 1>{}, integral_constant<int, -1>{}, yes{}, 0, integral_constant<int, S + 1>{}, no{}, no{}, 0);
  });

  // body of K step s (ring slot `slot` = s % NS): MORE = a further stage (s + NS) is requested, TAIL = it is the short one
  auto body = [&](int s, int slot, auto more_c, auto tail_c) {
    constexpr bool MORE = decltype(more_c)::value;
    const int nslot = slot + 1 == NS ? 0 : slot + 1;
    const bool new_chunk = KW::ENABLED && MORE && kw.starts(s + NS);
    if (new_chunk) kw.wait(s + NS);
    // stage s+1 must have landed; while requests continue, the NS-2 younger stages may stay in flight
    if constexpr (MORE) wait_vmcnt<(NS - 2) * LPW>(); else wait_vmcnt<0>();
    __syncthreads();
    if (new_chunk) kw.acquire();
    slice(integral_constant<int, (SL - 1) & 1>{}, integral_constant<int, 0>{}, yes{}, nslot, integral_constant<int, 0>{}, more_c, tail_c, slot);
    static_for<0, SL - 1>([&](auto sl_c) {
      constexpr int S = decltype(sl_c)::value;
      slice(integral_constant<int, S & 1>{}, integral_constant<int, S + 1>{}, yes{}, nslot, integral_constant<int, S + 1>{}, more_c, tail_c, slot);
    });
    if constexpr (MORE) {
      a_base += Cfg::BK * 2;
      b_base += b_step;
    }
  };
  int s = 0;
  const int n_main = nk - NS - (k_tail != 0 ? 1 : 0);   // K steps that request a whole further stage
  for (; s + NS <= n_main; s += NS)
    static_for<0, NS>([&](auto u_c) { body(s + decltype(u_c)::value, decltype(u_c)::value, yes{}, no{}); });
  int slot = 0;                                          // s is a multiple of NS here
  for (; s < n_main; s++) {
    body(s, slot, yes{}, no{});
    slot = slot + 1 == NS ? 0 : slot + 1;
  }
  if (k_tail != 0 && nk - NS - 1 >= 0) {                 // s == nk - NS - 1: this step requests the short last stage
    body(s, slot, yes{}, yes{});
    slot = slot + 1 == NS ? 0 : slot + 1;
    s++;
  }
  for (; s + 1 < nk; s++) {
    body(s, slot, no{}, no{});
    slot = slot + 1 == NS ? 0 : slot + 1;
  }
  slice(integral_constant<int, (SL - 1) & 1>{}, integral_constant<int, -1>{}, no{}, 0, integral_constant<int, 0>{}, no{}, no{}, 0);
  __syncthreads();  // all operand reads of this tile are complete: LDS is free for the epilogue

  // ---- epilogue.  Accumulator register e of lane l holds C[row = l%32][col = (e/4)*8 + (l/32)*4 + e%4] of its 32x32
  // block: stored from there, every store instruction would touch 32 rows with 16 bytes each.  Instead the wave
  // rounds its result to bf16 into an LDS region of its own and reads it back row-wise, so that a store instruction
  // writes whole 128-byte lines (16 bytes per lane, 8 lanes per row of a 64-wide wave tile).
  char* ep = smem + wave * (Cfg::WTM * Cfg::EP_PITCH);
  constexpr int OUT_WTN = Out::GATED ? Cfg::WTN / 2 : Cfg::WTN;  // output columns of the wave tile
#pragma unroll
  for (int mt = 0; mt < Cfg::MT; mt++) {
    const int row = mt * 32 + (lane & 31);
    float scale = 1.f;
    if (Out::SCALED && wm * Cfg::WTM + row < rows) out.row(wm * Cfg::WTM + row, scale);
    if constexpr (Out::GATED) {
      static_assert(!Out::GATED || Cfg::NT % 2 == 0, "gate and up blocks come in pairs");
#pragma unroll
      for (int np = 0; np < Cfg::NT / 2; np++) {
#pragma unroll
        for (int g = 0; g < 4; g++) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; e++) o[e] = (bf16_t)out.apply(acc[mt][2 * np][g * 4 + e], acc[mt][2 * np + 1][g * 4 + e]);
          *(bf16x4*)(ep + row * Cfg::EP_PITCH + (np * 32 + g * 8 + (lane >> 5) * 4) * 2) = o;
        }
      }
    } else {
#pragma unroll
      for (int nt = 0; nt < Cfg::NT; nt++) {
#pragma unroll
        for (int g = 0; g < 4; g++) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; e++) o[e] = (bf16_t)(Out::SCALED ? acc[mt][nt][g * 4 + e] * scale : acc[mt][nt][g * 4 + e]);
          *(bf16x4*)(ep + row * Cfg::EP_PITCH + (nt * 32 + g * 8 + (lane >> 5) * 4) * 2) = o;
        }
      }
    }
  }
  constexpr int EP_CPR = OUT_WTN / 8;                   // 16-byte chunks per row of the wave tile's output
  constexpr int EP_ITERS = Cfg::WTM * EP_CPR / 64;
  static_assert((Cfg::WTM * EP_CPR) % 64 == 0, "the epilogue hands out 16-byte chunks 64 at a time");
  const int out_cols = Out::GATED ? cols / 2 : cols;
  Out o = out;
#pragma unroll 4
  for (int i = 0; i < EP_ITERS; i++) {
    const int idx = i * 64 + lane;
    const int row = idx / EP_CPR, q = idx - row * EP_CPR;
    const int grow = wm * Cfg::WTM + row, col = wn * OUT_WTN + q * 8;
    o.group(wm * Cfg::WTM + (i * 64) / EP_CPR);
    if (grow < rows && col < out_cols) {  // cols % 8 == 0: a chunk is all in or all out
      o.store(grow, col, *(const u32x4*)(ep + row * Cfg::EP_PITCH + q * 16));
    }
  }
  // the next tile's loads overwrite the staging regions: all LDS reads must be done; the global stores need not be
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace tl
