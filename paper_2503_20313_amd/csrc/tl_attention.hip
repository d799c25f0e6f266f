// Sequence-parallel attention: AllGather of the K/V shards overlapped with flash attention of the local
// query shard (paper: "Kernel Design", AG KV + self-attention; background: sequence-parallel attention).
// gfx950 only, head_dim 128.
//
// One workgroup = one (head, block of 256 local queries); 8 waves, 32 queries each.  K/V blocks of 64 keys
// go through two LDS stages filled by direct-to-LDS loads.  Per wave and K/V block:
//   S^T[keys, q] = K . Q^T            (MFMA 32x32x16; K fragments from LDS, Q fragments live in registers)
//   online softmax down the key axis  (a lane owns one query column: the reduction over keys is over its own
//                                      registers plus one exchange with the lane 32 apart)
//   O^T[d, q]  += V^T . P^T           (P^T comes straight from the S^T accumulators: the key order inside an
//                                      MFMA's reduction is free, so V^T fragments are fetched in the order the
//                                      accumulators hold the keys, with transposing LDS reads)
// The first K/V block of every AllGather channel is preceded by consumer_tile_wait on that channel's K and V
// flags; a waiting workgroup works off producer tickets instead of idling.
#include "tl_ag_producer.h"
#include "tl_gemm_tile.h"
#include "tl_host.h"

namespace tl {

constexpr int kBQ = 256, kBKV = 64, kD = 128, kAttnWaves = 8, kAttnThreads = kAttnWaves * 64;
constexpr int kKvTileBytes = kBKV * kD * 2;            // 16 KiB
constexpr int kAttnLds = 2 * 2 * kKvTileBytes;         // two stages of (K tile, V tile)

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

__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32, 64); }

__global__ void __launch_bounds__(kAttnThreads) sp_attention_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __shared__ int s_ticket;
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform for the compiler too: the K/V loop holds barriers
  if ((int)blockIdx.x < p.n_comm) {
    // K and V producers share the communication workgroups: even ones start with K, odd ones with V
    if (blockIdx.x & 1) { ag_producer(p.vprod, tid, kAttnThreads, &s_ticket); ag_producer(p.kprod, tid, kAttnThreads, &s_ticket); }
    else { ag_producer(p.kprod, tid, kAttnThreads, &s_ticket); ag_producer(p.vprod, tid, kAttnThreads, &s_ticket); }
    return;
  }
  if (!p.do_compute) return;
  __builtin_amdgcn_s_setprio(TL_COMPUTE_WAVE_PRIO);  // matrix waves go first when they share a SIMD with communication waves
  // workgroup -> (head, query block): the query blocks of a head run on one die (workgroup w runs on die w % 8) so
  // that they share the head's K/V in that die's L2; heavy (late, for causal) query blocks first
  const int wid = blockIdx.x - p.n_comm;
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
  const int qw0 = q0 + wave * 32;                // first local query row of the wave
  const int g0 = p.rank * p.S_loc;               // global position of local row 0
  const long ldq = (long)p.heads * kD;           // row pitch of q/k/v/o in elements

  // ---- Q fragments (MFMA B operand): lane = query column l32, 8 consecutive d per 16-wide step
  bf16x8 qf[8];
  {
    int row = min(qw0 + l32, p.S_loc - 1);
    const bf16_t* qrow = p.q + (long)row * ldq + (long)head * kD + h * 8;
#pragma unroll
    for (int st = 0; st < 8; st++) qf[st] = *(const bf16x8*)(qrow + st * 16);
  }

  // ---- K/V stage loads: a tile is 64 rows x 256 bytes = 16 wave-wide loads of 1 KiB; wave w issues loads w and w+8
  // of the K tile and of the V tile.  LDS slot (row, pc) holds logical 16-byte chunk pc ^ f(row):
  //   K: f = row % 16   (fragment reads take one chunk from 16 consecutive rows)
  //   V: f = (row % 4) << 2 (transposing reads take 32 bytes from 4 consecutive rows)
  const int wg_q_hi = min(q0 + kBQ, p.S_loc) - 1;                 // last valid local query row of the workgroup
  const int n_kv = p.causal ? (g0 + wg_q_hi) / kBKV + 1 : (p.S + kBKV - 1) / kBKV;
  const char* kbase = (const char*)(p.kprod.gathered + (long)head * kD);
  const char* vbase = (const char*)(p.vprod.gathered + (long)head * kD);
  int ld_row[2], ld_kc[2], ld_vc[2];
#pragma unroll
  for (int i = 0; i < 2; i++) {
    int j = wave + i * kAttnWaves;
    int row = j * 4 + (lane >> 4), pc = lane & 15;
    ld_row[i] = row;
    ld_kc[i] = (pc ^ (row & 15)) * 16;
    ld_vc[i] = (pc ^ ((row & 3) << 2)) * 16;
  }
  auto issue_block = [&](int blk, int stage) {
    char* sk = smem + stage * 2 * kKvTileBytes;
    char* sv = sk + kKvTileBytes;
#pragma unroll
    for (int i = 0; i < 2; i++) {
      int j = wave + i * kAttnWaves;
      long row = min(blk * kBKV + ld_row[i], p.S - 1);
      lds_load16(kbase + row * ldq * 2 + ld_kc[i], sk + j * 1024);
      lds_load16(vbase + row * ldq * 2 + ld_vc[i], sv + j * 1024);
    }
  };
  // consumer_tile_wait on the K and V flags of the channel block `blk` starts, if it starts one
  auto wait_for_block = [&](int blk) {
    if (!p.do_wait) return;
    int row = blk * kBKV;
    if (row % p.rows_per_channel != 0) return;
    unsigned long long m = 1ull << (row / p.rows_per_channel);
    consumer_wait_or_produce(p.kprod, m, tid, kAttnThreads, &s_ticket);
    consumer_wait_or_produce(p.vprod, m, tid, kAttnThreads, &s_ticket);
  };

  // ---- per-lane LDS read offsets
  const int k_row_off = l32 * 256;                 // + t*32*256
  const int k_sw = l32 & 15;                       // (row % 16) is the same for both key tiles
  const int v_r = (lane & 15) >> 2;                // row inside the 4-row group a transposing read covers
  int v_off[4];                                    // per d-tile: address for (row v_r of a group, this lane's 4 columns)
#pragma unroll
  for (int dt = 0; dt < 4; dt++) {
    int col = dt * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    int c = (col >> 3) ^ (v_r << 2);
    v_off[dt] = v_r * 256 + c * 16 + (col & 4) * 2;
  }

  floatx16 oacc[4];
#pragma unroll
  for (int dt = 0; dt < 4; dt++)
#pragma unroll
    for (int e = 0; e < 16; e++) oacc[dt][e] = 0.f;
  float m_run = -1e30f, l_run = 0.f;
  const int q_glob = g0 + qw0 + l32;               // this lane's query position
  const int qw_glob_hi = g0 + min(qw0 + 31, p.S_loc - 1);

  for (int blk = -1; blk < n_kv; blk++) {
    wait_vmcnt<0>();
    __syncthreads();  // block blk has landed for every wave; nobody reads the other stage any more
    if (blk + 1 < n_kv) {
      wait_for_block(blk + 1);
      issue_block(blk + 1, (blk + 1) & 1);
    }
    if (blk < 0) continue;
    const int kv0 = blk * kBKV;
    if (p.causal && kv0 > qw_glob_hi) continue;    // every key of the block lies after every query of this wave
    const char* sk = smem + (blk & 1) * 2 * kKvTileBytes;
    const char* sv = sk + kKvTileBytes;

    // S^T = K . Q^T
    floatx16 sacc[2];
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int e = 0; e < 16; e++) sacc[t][e] = 0.f;
#pragma unroll
    for (int st = 0; st < 8; st++) {
#pragma unroll
      for (int t = 0; t < 2; t++) {
        bf16x8 kf = *(const bf16x8*)(sk + t * 32 * 256 + k_row_off + (((2 * st + h) ^ k_sw) << 4));
        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], sacc[t], 0, 0, 0);
      }
    }
    // scale, mask, online softmax.  Accumulator e of key tile t is key kv0 + t*32 + (e/4)*8 + h*4 + e%4.
    const bool need_mask = (p.causal && kv0 + kBKV - 1 > g0 + qw0) || kv0 + kBKV > p.S;
    // the softmax scale (times log2 e) is folded into the exponent: p = exp2(s*c - m*c) is one fused multiply-add and
    // one exp2 per score; the running maximum m is kept in units of the raw scores (c > 0)
    if (need_mask) {
#pragma unroll
      for (int t = 0; t < 2; t++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          int key = kv0 + t * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
          if ((p.causal && key > q_glob) || key >= p.S) sacc[t][e] = -INFINITY;
        }
    }
    float mloc = -1e30f;
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int e = 0; e < 16; e++) mloc = fmaxf(mloc, sacc[t][e]);
    mloc = fmaxf(mloc, xor32(mloc));
    const float m_new = fmaxf(m_run, mloc);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * p.scale_log2e);
    m_run = m_new;
    const float mc = -m_new * p.scale_log2e;
    float psum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int e = 0; e < 16; e++) {
        float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[t][e], p.scale_log2e, mc));
        psum += pv;
        pf[t * 2 + (e >> 3)][e & 7] = (bf16_t)pv;
      }
    l_run = l_run * alpha + psum;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {
#pragma unroll
      for (int dt = 0; dt < 4; dt++)
#pragma unroll
        for (int e = 0; e < 16; e++) oacc[dt][e] *= alpha;
    }
    // O^T += V^T . P^T.  Group g = 16 keys; MFMA reduction slot (h, j) of group g is key g*16 + (j/4)*8 + 4h + j%4,
    // i.e. the order in which pf[g] holds them: two transposing reads at key rows g*16 + 4h and g*16 + 8 + 4h.
#pragma unroll
    for (int g = 0; g < 4; g++) {
#pragma unroll
      for (int dt = 0; dt < 4; dt++) {
        const char* pv = sv + (g * 16 + 4 * h) * 256 + v_off[dt];
        short4_t lo = lds_read_tr(pv);
        short4_t hi = lds_read_tr(pv + 8 * 256);
        typedef short short8_t __attribute__((ext_vector_type(8)));
        short8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v), pf[g], oacc[dt], 0, 0, 0);
      }
    }
  }

  // ---- normalise and store: accumulator e of d-tile dt is d = dt*32 + (e/4)*8 + h*4 + e%4 of query l32
  const float l_tot = l_run + xor32(l_run);
  const float inv = 1.f / l_tot;
  const int row = qw0 + l32;
  if (row < p.S_loc) {
    bf16_t* orow = p.o + (long)row * ldq + (long)head * kD + h * 4;
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
      for (int gq = 0; gq < 4; gq++) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; e++) v[e] = (bf16_t)(oacc[dt][gq * 4 + e] * inv);
        *(bf16x4*)(orow + dt * 32 + gq * 8) = v;
      }
  }
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
  r->expected = r->rows_per_channel / Tm_p;
  r->n_comm = c.comm_workgroups > 0 ? c.comm_workgroups : (c.comm_mode == TL_COMM_WAVES ? 16 : 128);
  if (c.comm_mode == TL_COMM_NONE) r->n_comm = 0;
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
  if (int e = check_ctx(ctx)) return e;
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
  if (cfg.comm_mode == TL_COMM_STREAM || cfg.comm_mode == TL_COMM_EXTERNAL)
    return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: comm_mode must be NONE, WAVES or SIDE_KERNEL");

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
    TL_HIP(hipFuncSetAttribute((const void*)sp_attention_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kAttnLds));
    hipLaunchKernelGGL(sp_attention_kernel, dim3(grid), dim3(kAttnThreads), kAttnLds, cs, p);
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
  }
  return fail(TL_ERR_INVALID_ARG, "tl_sp_ag_attention: unknown comm_mode");
}

}  // extern "C"
