// Sequence-parallel attention: AllGather of the K/V shards overlapped with flash attention of the local
// query shard (paper: "Kernel Design", AG KV + self-attention; background: sequence-parallel attention).
// gfx950 only, head_dim 128.
//
// One workgroup = one (head, block of 256 local queries); a wave owns QT tiles of 32 queries (QT = 2: 4 waves, one
// per SIMD with the whole register file; QT = 1: 8 waves).  K/V blocks of 64 keys go through three LDS stages
// filled by direct-to-LDS loads.  Per wave, query tile and K/V block:
//   S^T[keys, q] = K . Q^T            (MFMA 32x32x16; K fragments from LDS, Q fragments live in registers)
//   online softmax down the key axis  (a lane owns one query column: the reduction over keys is over its own
//                                      registers plus one exchange with the lane 32 apart)
//   O^T[d, q]  += V^T . P^T           (P^T comes straight from the S^T accumulators: the key order inside an
//                                      MFMA's reduction is free, so V^T fragments are fetched in the order the
//                                      accumulators hold the keys, with transposing LDS reads)
// Every K or V fragment read from LDS feeds QT matrix instructions.  The first K/V block of every AllGather
// channel is preceded by consumer_tile_wait on that channel's K and V flags; a waiting workgroup works off
// producer tickets instead of idling.
#include "tl_ag_producer.h"
#include "tl_gemm_tile.h"
#include "tl_host.h"

namespace tl {

#ifndef TL_ATTN_QT
#define TL_ATTN_QT 1
#endif
#ifndef TL_ATTN_AHEAD
#define TL_ATTN_AHEAD 2
#endif
constexpr int kBQ = 256, kBKV = 64, kD = 128;
constexpr int kKvTileBytes = kBKV * kD * 2;            // 16 KiB
constexpr int kAttnLds = 3 * 2 * kKvTileBytes;         // three stages of (K tile, V tile)

struct AttnParams {
  AgProducer kprod, vprod;  // gathered K and V, each [S, heads*D]
  const bf16_t* q;          // [S_loc, heads, D]
  bf16_t* o;                // [S_loc, heads, D]
  int S, S_loc, heads, rank, causal;
  float scale_log2e;        // softmax scale * log2(e)
  int n_qblocks;
  int n_comm, do_compute, do_wait;
  int rows_per_channel, n_channels;  // AllGather channels along the sequence (per tensor)
};

// The two values a query column has in lanes l and l+32, in every lane (one VALU lane-half swap, no LDS round trip).
__device__ __forceinline__ void both_halves(float v, float& lo, float& hi) {
  const unsigned b = __builtin_bit_cast(unsigned, v);
  auto r = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  lo = __builtin_bit_cast(float, (unsigned)r[0]);
  hi = __builtin_bit_cast(float, (unsigned)r[1]);
}
// max(a, b) of two raw matrix-instruction results.  Written as a median with +inf, which the compiler turns into one
// v_max_f32 on the raw registers; fmaxf() on them would first canonicalise each operand with an instruction of its own.
__device__ __forceinline__ float raw_max(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, __builtin_inff()); }

// max(m, a, b) in one instruction on raw matrix-instruction results (finite or -inf)
__device__ __forceinline__ float raw_max3(float m, float a, float b) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(m), "v"(a), "v"(b));
  return r;
}

__device__ __forceinline__ float halves_max(float v) {
  float lo, hi;
  both_halves(v, lo, hi);
  return __builtin_fmaxf(lo, hi);
}

template <int QT>
__global__ void __launch_bounds__(512 / QT) sp_attention_kernel(const AttnParams p) {
  constexpr int NW = 8 / QT, NT = NW * 64;         // waves, threads
  constexpr int WQ = 32 * QT;                      // queries per wave
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int s_ticket;
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform for the compiler too: the K/V loop holds barriers
  if ((int)blockIdx.x < p.n_comm) {
    // K and V producers share the communication workgroups: even ones start with K, odd ones with V
    if (blockIdx.x & 1) { ag_producer(p.vprod, tid, NT, &s_ticket); ag_producer(p.kprod, tid, NT, &s_ticket); }
    else { ag_producer(p.kprod, tid, NT, &s_ticket); ag_producer(p.vprod, tid, NT, &s_ticket); }
    return;
  }
  if (!p.do_compute) return;
  __builtin_amdgcn_s_setprio(TL_COMPUTE_WAVE_PRIO);  // matrix waves go first when they share a SIMD with communication waves
  // workgroup -> (head, query block): the query blocks of a head run on one die (workgroup w runs on die w % 8) so
  // that they share the head's K/V in that die's L2; heavy (late, for causal) query blocks first
  const int wid = blockIdx.x - p.n_comm;
  const ClockSample cs0 = clock_sample_begin(wid);   // workgroup 0 has the heaviest query block: it runs for the whole kernel
  int head, qb;
  if (p.heads % kXcds == 0) {
    const int hpx = p.heads / kXcds, die = wid % kXcds, slot = wid / kXcds;
    head = die * hpx + slot % hpx;
    qb = p.n_qblocks - 1 - slot / hpx;
  } else {
    head = wid % p.heads;
    qb = p.n_qblocks - 1 - wid / p.heads;
  }
  const int q0 = qb * kBQ;                       // first local query row of the workgroup
  const int qw0 = q0 + wave * WQ;                // first local query row of the wave
  const int g0 = p.rank * p.S_loc;               // global position of local row 0
  const long ldq = (long)p.heads * kD;           // row pitch of q/k/v/o in elements

  // ---- Q fragments (MFMA B operand): lane = query column l32 of tile u, 8 consecutive d per 16-wide step
  bf16x8 qf[QT][8];
#pragma unroll
  for (int u = 0; u < QT; u++) {
    int row = min(qw0 + u * 32 + l32, p.S_loc - 1);
    const bf16_t* qrow = p.q + (long)row * ldq + (long)head * kD + h * 8;
#pragma unroll
    for (int st = 0; st < 8; st++) qf[u][st] = *(const bf16x8*)(qrow + st * 16);
  }

  // ---- K/V stage loads: a tile is 64 rows x 256 bytes = 16 wave-wide loads of 1 KiB; wave w issues loads w, w+NW, ..
  // of the K tile and of the V tile.  LDS slot (row, pc) holds logical 16-byte chunk pc ^ f(row):
  //   K: f = row % 16   (fragment reads take one chunk from 16 consecutive rows)
  //   V: f = (row % 4) << 2 (transposing reads take 32 bytes from 4 consecutive rows)
  constexpr int LPW = 16 / NW;                                    // loads per wave and tile
  const int wg_q_hi = min(q0 + kBQ, p.S_loc) - 1;                 // last valid local query row of the workgroup
  const int n_kv = p.causal ? (g0 + wg_q_hi) / kBKV + 1 : (p.S + kBKV - 1) / kBKV;
  // The global address of a load is a scalar base (the block's first row of this head, the same for every lane) plus a
  // lane offset that is fixed for the whole kernel: no vector arithmetic per block.  Every block is whole (the rows per
  // channel, and so S, are multiples of the block).
  const char* kbase = (const char*)(p.kprod.gathered + (long)head * kD);
  const char* vbase = (const char*)(p.vprod.gathered + (long)head * kD);
  unsigned ld_koff[LPW], ld_voff[LPW];
#pragma unroll
  for (int i = 0; i < LPW; i++) {
    int j = wave + i * NW;
    int row = j * 4 + (lane >> 4), pc = lane & 15;
    ld_koff[i] = (unsigned)row * (unsigned)(ldq * 2) + (unsigned)((pc ^ (row & 15)) * 16);
    ld_voff[i] = (unsigned)row * (unsigned)(ldq * 2) + (unsigned)((pc ^ ((row & 3) << 2)) * 16);
  }
  const unsigned smem_u = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)smem);
  auto issue_block = [&](int blk, int stage) __attribute__((always_inline)) {
    const long blk_off = (long)__builtin_amdgcn_readfirstlane(blk) * (kBKV * ldq * 2);
    const char* kb = (const char*)uniform64((unsigned long long)(kbase + blk_off));
    const char* vb = (const char*)uniform64((unsigned long long)(vbase + blk_off));
    const unsigned sk = smem_u + (unsigned)__builtin_amdgcn_readfirstlane(stage) * (2 * kKvTileBytes), sv = sk + kKvTileBytes;
#pragma unroll
    for (int i = 0; i < LPW; i++) {
      const int j = wave + i * NW;
      lds_load16_sbase(kb, ld_koff[i], sk + j * 1024);
      lds_load16_sbase(vb, ld_voff[i], sv + j * 1024);
    }
  };
  // consumer_tile_wait on the K and V flags of the channel block `blk` starts, if it starts one
  auto wait_for_block = [&](int blk) __attribute__((always_inline)) {
    if (!p.do_wait) return;
    int row = blk * kBKV;
    if (row % p.rows_per_channel != 0) return;
    if (p.do_wait == 2) {   // flags raised after copies of the runtime (no producer queue to help with): plain wait
      const int ch = row / p.rows_per_channel;
      if (tid == 0) {
        tile_wait(p.kprod.flags + ch, p.kprod.wait_target, p.kprod.ctl, ch);
        tile_wait(p.vprod.flags + ch, p.vprod.wait_target, p.vprod.ctl, p.n_channels + ch);
      }
      __syncthreads();
      return;
    }
    unsigned long long m = 1ull << (row / p.rows_per_channel);
    consumer_wait_or_produce(p.kprod, m, tid, NT, &s_ticket);
    consumer_wait_or_produce(p.vprod, m, tid, NT, &s_ticket);
  };

  // ---- per-lane LDS read offsets
  // K fragment i (k-step i/2, key tile i%2) of the K tile at byte offset kb = stage offset + this lane's row and
  // swizzle term: the chunk index (2*st + h) ^ (row % 16) only touches the low 8 address bits, so it is one XOR
  typedef short short8_t __attribute__((ext_vector_type(8)));
  const int k_lane_off = l32 * 256 + ((h ^ (l32 & 15)) << 4);
  auto kread = [&](int kb, int i) __attribute__((always_inline)) -> bf16x8 {
    return *(const bf16x8*)(smem + (i & 1) * 32 * 256 + (kb ^ ((i >> 1) << 5)));
  };
  // V^T fragment j (key group j/4 of 16 keys, d-tile j%4).  MFMA reduction slot (h, r) of group g is key
  // g*16 + (r/4)*8 + 4h + r%4, the order in which pf[.][g] holds the probabilities: two transposing reads at key
  // rows g*16 + 4h and g*16 + 8 + 4h.
  const int v_r = (lane & 15) >> 2;                // row inside the 4-row group a transposing read covers
  int v_off[4];                                    // per d-tile: address for (row v_r of a group, this lane's 4 columns)
#pragma unroll
  for (int dt = 0; dt < 4; dt++) {
    int col = dt * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    int c = (col >> 3) ^ (v_r << 2);
    v_off[dt] = (v_r + 4 * h) * 256 + c * 16 + (col & 4) * 2;
  }
  auto vread = [&](const char* sv, int j) __attribute__((always_inline)) -> bf16x8 {
    const char* pv = sv + (j >> 2) * 16 * 256 + v_off[j & 3];
    short4_t lo = lds_read_tr(pv);
    short4_t hi = lds_read_tr(pv + 8 * 256);
    return __builtin_bit_cast(bf16x8, (short8_t)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  floatx16 zero16;
#pragma unroll
  for (int e = 0; e < 16; e++) zero16[e] = 0.f;

  floatx16 oacc[QT][4];
#pragma unroll
  for (int u = 0; u < QT; u++)
#pragma unroll
    for (int dt = 0; dt < 4; dt++) oacc[u][dt] = zero16;
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int u = 0; u < QT; u++) { m_run[u] = -1e30f; l_run[u] = 0.f; }
  const int q_glob = g0 + qw0 + l32;               // this lane's query position in tile 0; tile u is 32u further
  const int qw_glob_hi = g0 + min(qw0 + WQ - 1, p.S_loc - 1);

  int st_cur = 0, st_nxt = 1, st_ld = 2;   // LDS stages of blocks blk, blk+1, blk+2
  // largest raw score of a query column in one block (both key tiles, both lane halves)
  auto block_max = [&](const floatx16 (&sc)[2]) __attribute__((always_inline)) -> float {
    float m = -1e30f;
#pragma unroll
    for (int e = 0; e < 16; e++) m = raw_max3(m, sc[0][e], sc[1][e]);
    return halves_max(m);
  };
  float m_blk[QT];   // block_max of the block the next iteration works on, computed one iteration early

  // One block of the software-pipelined loop: the scores of block blk are in c[u][key tile]; the scores of block
  // blk+1 go to n[u][key tile].  Iteration blk computes S(blk+1) while it takes block blk through the softmax, so
  // that the matrix pipe and the vector ALU of a SIMD work at the same time (all waves of the workgroup meet at a
  // barrier per block and would otherwise run the same phase side by side).  A K/V stage is live for three
  // iterations: filled during blk-2, K read during blk-1, V read during blk.
  auto block = [&](int blk, floatx16 (&c)[QT][2], floatx16 (&n)[QT][2]) __attribute__((always_inline)) {
    wait_vmcnt<0>();
    __syncthreads();  // block blk+1 has landed for every wave; nobody reads the stage of block blk-1 any more
    if (blk + 2 < n_kv) {
      wait_for_block(blk + 2);
      issue_block(blk + 2, st_ld);
    }
    const int kv0 = blk * kBKV;
    // a block whose keys all lie after every query of this wave is skipped, and so are all later ones
    if (!(p.causal && kv0 > qw_glob_hi)) {
      // the first K fragments of block blk+1 are on their way while part 1 of the softmax runs
      const int kb = st_nxt * 2 * kKvTileBytes + k_lane_off;
      const char* sv = smem + st_cur * 2 * kKvTileBytes + kKvTileBytes;
      constexpr int RD = TL_ATTN_AHEAD, RN = RD + 1;   // fragments read ahead, ring size
      bf16x8 fr[RN];
#pragma unroll
      for (int i = 0; i < RD; i++) fr[i] = kread(kb, i);
      __builtin_amdgcn_sched_barrier(0);
      // mask.  Accumulator e of key tile t is key kv0 + t*32 + (e/4)*8 + h*4 + e%4.  A query tile whose keys are all
      // masked keeps its running maximum (finite from block 0 on) and gets probabilities exp2(-inf) = 0.
      const bool need_mask = (p.causal && kv0 + kBKV - 1 > g0 + qw0) || kv0 + kBKV > p.S;
      if (need_mask) {
#pragma unroll
        for (int u = 0; u < QT; u++)
#pragma unroll
          for (int t = 0; t < 2; t++)
#pragma unroll
            for (int e = 0; e < 16; e++) {
              int key = kv0 + t * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
              if ((p.causal && key > q_glob + u * 32) || key >= p.S) c[u][t][e] = -INFINITY;
            }
      }
      // online softmax, part 1: running maximum and the rescaling of O.  The softmax scale (times log2 e) is folded
      // into the exponent: p = exp2(s*c - m*c) is one fused multiply-add and one exp2 per score; the running
      // maximum m is kept in units of the raw scores (c > 0)
      float alpha[QT], mc[QT];
      bool rescale = false;
      if (need_mask) {
#pragma unroll
        for (int u = 0; u < QT; u++) m_blk[u] = block_max(c[u]);
      }
#pragma unroll
      for (int u = 0; u < QT; u++) {
        const float m_new = fmaxf(m_run[u], m_blk[u]);
        alpha[u] = __builtin_amdgcn_exp2f((m_run[u] - m_new) * p.scale_log2e);
        m_run[u] = m_new;
        mc[u] = -m_new * p.scale_log2e;
        rescale |= alpha[u] != 1.f;
      }
      if (__builtin_amdgcn_ballot_w64(rescale)) {
#pragma unroll
        for (int u = 0; u < QT; u++)
#pragma unroll
          for (int dt = 0; dt < 4; dt++)
#pragma unroll
            for (int e = 0; e < 16; e++) oacc[u][dt][e] *= alpha[u];
      }
      // ---- 32 fragments in a fixed issue order, each feeding QT matrix instructions: 16 of S(blk+1) = K.Q^T (past
      // the last block: of whatever the stage holds; the result is dropped), then 16 of O^T += V^T.P^T.  Fragments
      // are read from LDS two ahead, and each instruction slot carries a slice of part 2 of the softmax
      // (p = exp2(s*c - m*c), row sum, conversion to the bf16 operand).  The scores are taken key group by key
      // group (16 keys), query tile by query tile; score y of that order is done in slot y*7/8, so that the
      // probabilities of key group g are complete before the first slot that multiplies them, (16 + 4g)*QT.
      bf16x8 pf[QT][4];
      float psum[QT], m_part[QT], m_next[QT];
#pragma unroll
      for (int u = 0; u < QT; u++) psum[u] = 0.f;
      static_for<0, 32 * QT>([&](auto s_c) {
        constexpr int sl = decltype(s_c)::value, f = sl / QT, u = sl % QT;
        if constexpr (u == 0) {
          if constexpr (f + RD < 16) fr[(f + RD) % RN] = kread(kb, f + RD);
          else if constexpr (f + RD < 32) fr[(f + RD) % RN] = vread(sv, f + RD - 16);
        }
        if constexpr (f < 16) {
          floatx16& acc = n[u][f & 1];
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[f % RN], qf[u][f >> 1], f < 2 ? zero16 : acc, 0, 0, 0);
        } else {
          constexpr int j = f - 16;
          oacc[u][j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[f % RN], pf[u][j >> 2], oacc[u][j & 3], 0, 0, 0);
        }
        // the maximum of block blk+1's scores, ready for the next iteration (a masked block recomputes it after masking)
        if constexpr (f >= 18 && f < 18 + 4 && u == 0) {
          constexpr int q = f - 18;   // quarter of the 16 accumulator pairs
#pragma unroll
          for (int uu = 0; uu < QT; uu++) {
            float m = q == 0 ? -1e30f : m_part[uu];
#pragma unroll
            for (int e = q * 4; e < q * 4 + 4; e++) m = raw_max3(m, n[uu][0][e], n[uu][1][e]);
            m_part[uu] = m;
          }
        }
        if constexpr (f == 23 && u == 0) {
#pragma unroll
          for (int uu = 0; uu < QT; uu++) m_next[uu] = halves_max(m_part[uu]);
        }
        static_for<0, 32 * QT>([&](auto y_c) {
          constexpr int y = decltype(y_c)::value;
          if constexpr (y * 7 / 8 == sl) {
            constexpr int g = y / (8 * QT), uu = (y / 8) % QT, i = y % 8;
            const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(c[uu][g >> 1][(g & 1) * 8 + i], p.scale_log2e, mc[uu]));
            pf[uu][g][i] = (bf16_t)pv;
            // the row sum takes the unrounded probabilities, one plain addition each.  (A dot product of the packed pair with
            // (1, 1) is one instruction for two values, but v_dot2c_f32_bf16 runs in the matrix pipeline: measured, each one
            // holds up the matrix instructions for 16 cycles, whereas additions issue beside them.)
            psum[uu] += pv;
          }
        });
        __builtin_amdgcn_sched_barrier(0);
      });
#pragma unroll
      for (int u = 0; u < QT; u++) {
        l_run[u] = l_run[u] * alpha[u] + psum[u];
        m_blk[u] = m_next[u];
      }
    }
    const int st_free = st_cur;
    st_cur = st_nxt; st_nxt = st_ld; st_ld = st_free;
  };

  for (int b = 0; b < 2 && b < n_kv; b++) {
    wait_for_block(b);
    issue_block(b, b);
  }
  wait_vmcnt<0>();
  __syncthreads();
  floatx16 sa[QT][2], sb[QT][2];   // scores of even blocks / of odd blocks
#pragma unroll
  for (int i = 0; i < 16; i++) {
    bf16x8 kf = kread(k_lane_off, i);
#pragma unroll
    for (int u = 0; u < QT; u++)
      sa[u][i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[u][i >> 1], i < 2 ? zero16 : sa[u][i & 1], 0, 0, 0);
  }
#pragma unroll
  for (int u = 0; u < QT; u++) m_blk[u] = block_max(sa[u]);
  for (int blk = 0; blk < n_kv; blk += 2) {
    block(blk, sa, sb);
    if (blk + 1 < n_kv) block(blk + 1, sb, sa);
  }

  // ---- normalise and store: accumulator e of d-tile dt is d = dt*32 + (e/4)*8 + h*4 + e%4 of query l32 of tile u
#pragma unroll
  for (int u = 0; u < QT; u++) {
    float l_lo, l_hi;
    both_halves(l_run[u], l_lo, l_hi);
    const float l_tot = l_lo + l_hi;
    const float inv = 1.f / l_tot;
    const int row = qw0 + u * 32 + l32;
    if (row < p.S_loc) {
      bf16_t* orow = p.o + (long)row * ldq + (long)head * kD + h * 4;
#pragma unroll
      for (int dt = 0; dt < 4; dt++)
#pragma unroll
        for (int gq = 0; gq < 4; gq++) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; e++) v[e] = (bf16_t)(oacc[u][dt][gq * 4 + e] * inv);
          *(bf16x4*)(orow + dt * 32 + gq * 8) = v;
        }
    }
  }
  clock_sample_end(cs0, wid, p.kprod.ctl.status);
}

constexpr int kAttnQT = TL_ATTN_QT, kAttnThreads = 512 / kAttnQT;

// rank_notify for a shard copied by the runtime: raise `count` consecutive channel flags by one.
__global__ void kv_notify_kernel(unsigned* flags, int count) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) tile_notify(flags + i, 1u);
}

__global__ void __launch_bounds__(256) kv_producer_kernel(const AgProducer k, const AgProducer v) {
  __shared__ int s_ticket;
  if (blockIdx.x & 1) { ag_producer(v, threadIdx.x, 256, &s_ticket); ag_producer(k, threadIdx.x, 256, &s_ticket); }
  else { ag_producer(k, threadIdx.x, 256, &s_ticket); ag_producer(v, threadIdx.x, 256, &s_ticket); }
}

struct AttnResolved {
  int S_loc, n_qblocks, C, rows_per_channel, Tm_p, n_ptm, expected, n_comm, shards_needed;
};

static int resolve_attn(const tl_ctx* ctx, int S, int heads, int head_dim, int causal, AttnResolved* r) {
  const tl_config& c = ctx->cfg;
  const int R = c.world_size;
  if (S <= 0 || heads <= 0) return fail(TL_ERR_INVALID_ARG, "S and heads must be positive");
  if (head_dim != kD) return fail(TL_ERR_UNSUPPORTED_SHAPE, "head_dim %d is not supported (128 only)", head_dim);
  if (S % R) return fail(TL_ERR_UNSUPPORTED_SHAPE, "world size %d must divide S=%d", R, S);
  memset(r, 0, sizeof *r);
  r->S_loc = S / R;
  r->C = c.channels_per_rank;
  if (r->S_loc % r->C || (r->S_loc / r->C) % kBKV)
    return fail(TL_ERR_UNSUPPORTED_SHAPE, "the rows per channel S/(R*C)=%d/%d must be a multiple of %d", r->S_loc, r->C, kBKV);
  if (R * r->C > 64) return fail(TL_ERR_UNSUPPORTED_SHAPE, "at most 64 AllGather channels per tensor (R*C=%d)", R * r->C);
  r->rows_per_channel = r->S_loc / r->C;
  r->n_qblocks = ceil_div(r->S_loc, kBQ);
  int Tm_p = c.comm_tile_m;
  if (Tm_p == 0) {
    Tm_p = r->rows_per_channel;
    while (Tm_p > 32 && Tm_p % 2 == 0) Tm_p /= 2;
  }
  if (Tm_p <= 0 || r->rows_per_channel % Tm_p) return fail(TL_ERR_UNSUPPORTED_SHAPE, "producer row tile %d must divide S/(R*C)=%d", Tm_p, r->rows_per_channel);
  r->Tm_p = Tm_p;
  r->shards_needed = causal ? c.rank + 1 : R;   // causal: keys after this rank's positions are never read
  r->n_ptm = r->shards_needed * (r->S_loc / Tm_p);
  r->expected = c.comm_mode == TL_COMM_COPY_ENGINE ? 1 : r->rows_per_channel / Tm_p;   // one notification per channel after a shard's copy
  r->n_comm = c.comm_workgroups > 0 ? c.comm_workgroups : (c.comm_mode == TL_COMM_WAVES ? 16 : 128);
  if (c.comm_mode == TL_COMM_NONE || c.comm_mode == TL_COMM_COPY_ENGINE) r->n_comm = 0;
  return TL_OK;
}

}  // namespace tl

using namespace tl;

extern "C" {

int tl_attn_query(const tl_ctx* ctx, int S, int heads, int head_dim, int causal, int* info) {
  if (int e = check_ctx(ctx)) return e;
  if (!info) return fail(TL_ERR_INVALID_ARG, "info must not be null");
  AttnResolved r;
  if (int e = resolve_attn(ctx, S, heads, head_dim, causal, &r)) return e;
  int v[8] = {kBQ, kBKV, 2 * ctx->cfg.world_size * r.C, 256, r.expected, r.shards_needed, r.n_qblocks * heads, r.n_comm};
  memcpy(info, v, sizeof v);
  return TL_OK;
}

int tl_sp_ag_attention(tl_ctx* ctx, const void* q, const void* const* k_shards, const void* const* v_shards, void* k_gathered,
                       void* v_gathered, void* o, int S, int heads, int head_dim, int causal, float scale, unsigned* flags, unsigned epoch,
                       void* workspace, size_t ws_bytes, void* compute_stream, void* comm_stream) {
  if (int e = check_op_ctx(ctx)) return e;
  const tl_config& cfg = ctx->cfg;
  if (!q || !k_shards || !v_shards || !k_gathered || !v_gathered || !o || !flags || !workspace) return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: null pointer argument");
  if (epoch == 0) return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: epoch starts at 1");
  if (!(scale > 0.f)) return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: scale must be positive");
  AttnResolved r;
  if (int e = resolve_attn(ctx, S, heads, head_dim, causal, &r)) return e;
  if (ws_bytes < 256) return fail(TL_ERR_WORKSPACE_TOO_SMALL, "tl_sp_ag_attention: workspace of %zu bytes, 256 needed", ws_bytes);
  const int R = cfg.world_size;
  if (!aligned16(q) || !aligned16(k_gathered) || !aligned16(v_gathered) || !aligned16(o)) return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: device pointers must be 16-byte aligned");
  for (int s = 0; s < R; s++)
    if (!k_shards[s] || !v_shards[s] || !aligned16(k_shards[s]) || !aligned16(v_shards[s]))
      return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: k_shards[%d] or v_shards[%d] is null or misaligned", s, s);
  // (TL_COMM_STREAM is not offered: the runtime's copy kernels would have to become resident beside attention workgroups
  // that hold every compute unit while they wait for exactly those copies)
  if (cfg.comm_mode == TL_COMM_STREAM || cfg.comm_mode == TL_COMM_EXTERNAL)
    return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: comm_mode must be NONE, WAVES, SIDE_KERNEL or COPY_ENGINE");
  if (cfg.comm_mode == TL_COMM_COPY_ENGINE && cfg.link_gbps > 0)
    return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: simulated links need the library's own producers (WAVES or SIDE_KERNEL)");

  AttnParams p;
  memset(&p, 0, sizeof p);
  const int ld = heads * head_dim;
  const int RC = R * r.C;
  fill_ag_producer(ctx, &p.kprod, k_shards, k_gathered, ld, r.Tm_p, ld, r.n_ptm, 1, r.S_loc, r.rows_per_channel, flags, epoch, workspace);
  fill_ag_producer(ctx, &p.vprod, v_shards, v_gathered, ld, r.Tm_p, ld, r.n_ptm, 1, r.S_loc, r.rows_per_channel, flags + RC, epoch, workspace);
  // keys are consumed from position 0 upwards: the queue starts with rank 0's shard
  p.kprod.first_src = 0; p.vprod.first_src = 0;
  p.kprod.n_ptm_all = p.vprod.n_ptm_all = R * (r.S_loc / r.Tm_p);
  p.vprod.ticket = (unsigned*)workspace + 2;  // word 1: K queue, word 2: V queue
  p.kprod.pace_q8 *= 2; p.vprod.pace_q8 *= 2;  // K and V of a rank share its link
  p.kprod.wait_target = p.vprod.wait_target = epoch * (unsigned)r.expected;
  p.q = (const bf16_t*)q;
  p.o = (bf16_t*)o;
  p.S = S; p.S_loc = r.S_loc; p.heads = heads; p.rank = cfg.rank; p.causal = causal ? 1 : 0;
  p.scale_log2e = scale * 1.4426950408889634f;
  p.n_qblocks = r.n_qblocks;
  p.rows_per_channel = r.rows_per_channel;
  p.n_channels = RC;
  hipStream_t cs = (hipStream_t)compute_stream, ms = (hipStream_t)comm_stream;
  const bool alone = cfg.comm_alone != 0;
  p.do_compute = alone ? 0 : 1;
  const int n_wg = r.n_qblocks * heads;
  auto launch = [&](int grid) -> int {
    TL_HIP(hipFuncSetAttribute((const void*)sp_attention_kernel<kAttnQT>, hipFuncAttributeMaxDynamicSharedMemorySize, kAttnLds));
    hipLaunchKernelGGL(sp_attention_kernel<kAttnQT>, dim3(grid), dim3(kAttnThreads), kAttnLds, cs, p);
    TL_HIP(hipGetLastError());
    return TL_OK;
  };
  switch (cfg.comm_mode) {
    case TL_COMM_NONE:
      if (alone) return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: comm_alone needs a producer");
      p.n_comm = 0; p.do_wait = 0;
      return launch(n_wg);
    case TL_COMM_WAVES:
      p.n_comm = r.n_comm; p.do_wait = 1;
      return launch(alone ? r.n_comm : n_wg + r.n_comm);
    case TL_COMM_SIDE_KERNEL:
      p.n_comm = 0; p.do_wait = 1;
      hipLaunchKernelGGL(kv_producer_kernel, dim3(r.n_comm), dim3(256), 0, ms, p.kprod, p.vprod);
      TL_HIP(hipGetLastError());
      return alone ? TL_OK : launch(n_wg);
    case TL_COMM_COPY_ENGINE: {
      // rank_copy_data + rank_notify per source rank on the communication stream, in the order the keys are consumed:
      // the copy kind that keeps the compute units out of it (the runtime hands it to a copy engine), then a small
      // kernel that raises the shard's K (or V) channel flags
      p.n_comm = 0; p.do_wait = 2;
      p.kprod.wait_target = p.vprod.wait_target = epoch;
      const size_t shard_bytes = (size_t)r.S_loc * ld * sizeof(bf16_t);
      for (int s = 0; s < r.shards_needed; s++) {
        TL_HIP(hipMemcpyAsync((char*)k_gathered + (size_t)s * shard_bytes, k_shards[s], shard_bytes, hipMemcpyDeviceToDeviceNoCU, ms));
        hipLaunchKernelGGL(kv_notify_kernel, dim3((r.C + 63) / 64), dim3(64), 0, ms, flags + s * r.C, r.C);
        TL_HIP(hipMemcpyAsync((char*)v_gathered + (size_t)s * shard_bytes, v_shards[s], shard_bytes, hipMemcpyDeviceToDeviceNoCU, ms));
        hipLaunchKernelGGL(kv_notify_kernel, dim3((r.C + 63) / 64), dim3(64), 0, ms, flags + RC + s * r.C, r.C);
        TL_HIP(hipGetLastError());
      }
      return alone ? TL_OK : launch(n_wg);
    }
  }
  return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: unknown comm_mode");
}

}  // extern "C"
