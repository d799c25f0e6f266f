/*
 * tilelink_mi355 — tile-centric overlapped tensor-parallel operators for one MI355X (gfx950).
 *
 * C ABI.  Every operator is one GPU's share of a tensor-parallel layer over `world_size`
 * ranks: the other ranks' shards and partial results are ordinary device buffers the caller
 * has filled (there is no second GPU and no collective library involved).
 *
 * Conventions that hold for every entry point
 *   - Return value: TL_OK (0) or a negative tl_status.  tl_last_error() returns a
 *     thread-local, human-readable description of the most recent failure.
 *   - "dev" pointers are device (HBM) addresses owned by the caller; "host" pointers are
 *     ordinary host memory.  The library never frees caller memory and allocates no device
 *     memory in an operator call.
 *   - bf16 tensors are row-major arrays of 16-bit bfloat16; all leading dimensions are
 *     dense (no padding between rows).
 *   - Calls are asynchronous: work is enqueued on the caller's streams (hipStream_t passed
 *     as void*; NULL = the default stream) and the caller synchronises.  Arguments are
 *     validated before anything is enqueued.
 *   - Barrier flags are `unsigned` counters in device memory that only ever grow.  The
 *     caller zeroes them once; call number `epoch` (1, 2, 3, ...) waits for
 *     `epoch * expected`, so no reset is needed between calls.  Reusing a flag array for
 *     a call with a different geometry requires zeroing it again.
 *   - A bounded wait that expires (tl_config.spin_timeout_us) writes a non-zero code into
 *     the first word of the workspace and lets the kernel finish with undefined output;
 *     tl_check_status() reports it as TL_ERR_TIMEOUT.
 *
 * Notation follows the paper: R = world size, r = rank, C = channels (barriers) per rank,
 * producer tile Tm_p x Tn_p, consumer (compute) tile Tm_c x Tn_c.
 */
#ifndef TILELINK_MI355_H
#define TILELINK_MI355_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tl_status {
  TL_OK = 0,
  TL_ERR_INVALID_ARG = -1,       /* null pointer, non-positive size, rank outside [0,R) ... */
  TL_ERR_UNSUPPORTED_SHAPE = -2, /* a divisibility rule of the mapping or of the kernel is violated */
  TL_ERR_WORKSPACE_TOO_SMALL = -3,
  TL_ERR_HIP = -4,               /* a HIP runtime call failed; message holds hipGetErrorString */
  TL_ERR_TIMEOUT = -5            /* a bounded flag wait expired (reported by tl_check_status) */
} tl_status;

/* Resource binding of the communication side (paper: "Decoupled Design Space"). */
enum { TL_COMM_NONE = 0,   /* data already in place: no producer runs, consumers do not wait */
       TL_COMM_WAVES = 1,  /* device-side: dedicated copy/reduce workgroups inside the fused kernel
                              (tile_pull_data / tile_push_data + *_tile_notify) */
       TL_COMM_STREAM = 2, /* host-side: copies and notifications enqueued on comm_stream through the runtime's
                              copy path (rank_copy_data + rank_notify); reduce work runs as a second kernel there */
       TL_COMM_SIDE_KERNEL = 3, /* device-side copy/reduce workgroups launched as a small-footprint kernel of their
                              own on comm_stream, so that they can share compute units with resident GEMM workgroups */
       TL_COMM_EXTERNAL = 4, /* consumers wait on the flags but the library runs no producer: the caller (a peer,
                              another library) moves the data and raises the flags itself */
       TL_COMM_COPY_ENGINE = 5 /* tl_ag_gemm family: as TL_COMM_STREAM, but every shard copy is handed to a copy (DMA) engine,
                              which occupies no compute unit (rank_copy_data on the copy engine, the binding the paper's
                              evaluation uses for the AllGather of the MLP layer); a one-wave kernel behind each copy
                              raises the shard's flags (rank_notify).  The GEMM grid keeps every compute unit. */ };

/* Tile order of the compute side. */
enum { TL_ORDER_NATURAL = 0, /* row-major over (row block, column block) */
       TL_ORDER_RING = 1,    /* row blocks rotated by owner rank: AG+GEMM starts with the local
                                shard's rows, GEMM+RS starts with rank r+1's segment and ends with its own */
       TL_ORDER_OWN_FIRST = 2, /* as RING, but GEMM+RS starts with its own segment and then follows the ring */
       TL_ORDER_ARRIVAL = 3    /* tl_ag_gemm: the local shard's row blocks, then row block j of every other rank along
                                  the ring before row block j+1 of any -- the order in which links that run side by
                                  side deliver -- and the producer queue in the same order (needs whole row blocks per
                                  rank, else RING).  The other operators treat it as OWN_FIRST. */ };

/* Operators, for tl_query_workspace / tl_dump_schedule. */
enum { TL_OP_AG_GEMM = 0, TL_OP_GEMM_RS = 1, TL_OP_MOE_AG_GATHER_GEMM = 2, TL_OP_MOE_GEMM_SCATTER_RS = 3,
       TL_OP_SP_AG_ATTENTION = 4 };

/* The mapping context (the paper's BlockChannel: rank, world size, barrier configuration,
 * producer/consumer tile relationship) plus the free choices of the decoupled design space.
 * A field set to 0 selects the library default for the shape at hand. */
typedef struct tl_config {
  int world_size;          /* R >= 1 */
  int rank;                /* r in [0, R) */
  int channels_per_rank;   /* C >= 1; barriers per source rank */
  int tile_m, tile_n;      /* consumer tile Tm_c x Tn_c; supported pairs: 256x256, 256x224, 128x128 (0 = auto) */
  int comm_tile_m;         /* producer row-tile Tm_p (AllGather) / reduce row-tile (ReduceScatter); 0 = auto */
  int comm_tile_n;         /* producer column-tile Tn_p; 0 = whole row */
  int comm_mode;           /* TL_COMM_* */
  int comm_workgroups;     /* workgroups given to communication in TL_COMM_WAVES (paper's examples: 20 SMs); 0 = auto */
  int compute_workgroups;  /* persistent compute workgroups G; 0 = number of compute units */
  int tile_order;          /* TL_ORDER_* */
  int xcd_swizzle;         /* 1: workgroups on one die take neighbouring tiles (see tl_dump_schedule) */
  int group_m;             /* row blocks walked together in the compute order (column block slowest inside a group); 0 = auto */
  unsigned spin_timeout_us;/* bound on every flag wait; 0 = unbounded */
  int comm_alone;          /* 1: run only the communication side of comm_mode (no GEMM tiles; producer-consumer waits
                              skipped, the GEMM's output is taken as already complete): for timing */
  int rs_direct_push;      /* ReduceScatter operators: 1 = the stage that produces the partial result stores the rows of
                              other ranks' segments straight into peer_push[] (tile_push_data from the producer's
                              epilogue) and only the rows of the own segment into `partial`; the communication side then
                              just forwards the notification for those tiles instead of copying them.  The flags keep
                              their meaning; the rows of `partial` outside the own segment are not written.
                              2 (tl_gemm_rs only; 1 elsewhere) = in addition the GEMM epilogue reduces the rows of the own
                              segment itself: it waits for the peers' contributions (peer_tile_wait) before such a tile and
                              writes `out` together with the own rows of `partial`; same arithmetic, same bits as 1. */
  int ag_k_chunks;         /* tl_ag_gemm: >= 2 cuts every AllGather channel into that many chunks along K, each with a
                              barrier of its own (flag index channel*ag_k_chunks + chunk); the producer tile is then
                              comm_tile_m x K/ag_k_chunks and the queue delivers chunk 0 of all rows before chunk 1.  A
                              GEMM tile starts as soon as the first chunk of its rows is there and waits for each
                              further chunk when its K loop reaches it (the decoupled tile sizes of the paper's
                              "tile size" sub-space, applied along K).  Needs K divisible by 64*ag_k_chunks with at
                              least 8 K steps of 64 per chunk, comm_tile_n 0, and TL_COMM_WAVES or TL_COMM_SIDE_KERNEL
                              with the 256x256 compute tile; elsewhere, and for 0 or 1, one flag per channel. */
  int link_gbps;           /* AllGather operators: 0 = the producers copy as fast as they can.  > 0 = simulated links: every
                              other rank's shard arrives at this many GB/s (decimal), all ranks side by side, starting
                              when the call's first producer starts; a producer tile of a remote shard is not copied
                              before its last byte would have arrived, and the queue takes row tile j of every remote
                              rank before row tile j+1 of any.  xGMI: 153.  Results are unchanged. */
} tl_config;

typedef struct tl_ctx tl_ctx;

/* Creates a context for the current HIP device from *cfg (copied).  Host call. */
int tl_ctx_create(const tl_config* cfg /*host*/, tl_ctx** out /*host*/);
/* A context for the host-side queries only (tl_query_workspace, tl_resolve, tl_dump_schedule, tl_moe_query,
 * tl_attn_query): no HIP call is made, `num_compute_units` stands for the device's compute-unit count (MI355X: 256).
 * Every call that would enqueue GPU work returns TL_ERR_INVALID_ARG for such a context.  For planning on a machine
 * without a GPU and for checking the mapping tables (paper: "Tile-Centric Mapping") on the CPU. */
int tl_ctx_create_host(const tl_config* cfg /*host*/, int num_compute_units, tl_ctx** out /*host*/);
int tl_ctx_destroy(tl_ctx* ctx);
const char* tl_last_error(void);
/* Library version string and the offload architecture it was built for. */
const char* tl_version(void);

/* Bytes of workspace and number of flag words operator `op` needs for `dims`
 * (AG_GEMM, GEMM_RS: {M,N,K}; MoE: {T,H,I,E,topk}; attention: {S,heads,head_dim}).  Host call, no GPU work. */
int tl_query_workspace(const tl_ctx* ctx, int op, const long long* dims /*host*/, size_t* ws_bytes /*host*/,
                       size_t* n_flags /*host*/);

/* Synchronous: copies the status word out of `workspace` (after the caller synchronised the
 * streams) and returns TL_OK or TL_ERR_TIMEOUT; clears the word.  workspace = NULL: the static scratch of
 * tl_ag_gemm_static on the context's device. */
int tl_check_status(tl_ctx* ctx, void* workspace /*dev*/);

/* Measurement aid: the rate the matrix cores alone sustain on given operand data (an MFMA-only register loop, one
 * workgroup of 8 waves per compute unit; no LDS, no loads inside the loop).  Enqueues one kernel on `stream`.
 *   operands  dev, bf16 values drawn as the GEMM inputs are (num_compute_units * 512 * 48 of them, 16-byte aligned);
 *             operand_bytes = their size, checked.   iters = loop iterations of 8 matrix instructions per wave.
 *   sink      dev float[num_compute_units * 512] (written; keeps the loop alive)
 *   clocks    dev long long[2] (written): shader cycles and 100 MHz ticks the first workgroup's loop took
 *   flop      host, optional: the matrix work of the launch, so that flop / measured time = the sustained rate. */
int tl_mfma_peak_probe(tl_ctx* ctx, const void* operands /*dev*/, size_t operand_bytes, int iters, float* sink /*dev*/,
                       long long* clocks /*dev*/, void* stream, double* flop /*host*/);

/* Measurement aid: what a SIMD issues beside a running matrix instruction.  Enqueues on `stream` a kernel of one 512-thread
 * workgroup per compute unit (two waves per SIMD) whose waves run `iters` x 8 slots; a slot is one 32x32x16 bf16 matrix
 * instruction (left out if with_mfma == 0) followed by the vector instructions of `mode`: 0 none, 1 six v_fma_f32, 2 two
 * v_exp_f32, 3 v_cvt_pk_bf16_f32 + v_max3_f32, 4 one v_dot2c_f32_bf16.  All operands are zero, so the chip's power limit
 * plays no part and the clock stays at its maximum: the caller times the launch (events on `stream`) and compares modes.
 *   sink dev float[1 + num_compute_units * 512] (sink[0] is read, all are written); clocks dev long long[2] (cycles and
 *   100 MHz ticks of the first workgroup); *slots (host, optional) = slots per wave.  No paper passage defines this. */
int tl_issue_probe(tl_ctx* ctx, int with_mfma, int mode, int iters, float* sink /*dev*/, long long* clocks /*dev*/, void* stream,
                   double* slots /*host*/);

/* Measurement aid.  Synchronous: after a tl_ag_gemm-family, tl_gemm_rs-family or tl_sp_ag_attention call has completed, out[0] = shader-clock
 * cycles and out[1] = ticks of the 100 MHz wall clock during which the call's first compute workgroup was resident
 * (kept in bytes 32..47 of the workspace): out[0] / out[1] x 100 is the shader clock in MHz the tile kernel ran at.  On
 * this chip that clock depends on the operand data, so it belongs beside every throughput figure.  workspace = NULL: the
 * static scratch of tl_ag_gemm_static. */
int tl_read_clocks(tl_ctx* ctx, void* workspace /*dev*/, long long* out /*host, 2 values*/);

/*
 * AllGather + GEMM (paper: "Tile-Centric Mapping", AllGather pull mode + GEMM; tensor-parallel
 * FFN first half).  C[M,N] = concat_rows(a_shards[0..R-1])[M,K] . B[K,N], fp32 accumulation,
 * bf16 output rounded to nearest even.
 *   a_shards   host array of R dev pointers, shard q = rows [q*M/R, (q+1)*M/R) of A, each [M/R, K] bf16.
 *              If a_shards[r] == a_gathered + r*(M/R)*K the local shard is taken in place.
 *   a_gathered dev [M,K] bf16: written by the producer, read by the GEMM tiles.
 *   b          dev [K,N] bf16.           c  dev [M,N] bf16 (written).
 *   flags      dev unsigned[R*C]; channel index = src_rank*C + local channel (the global index of the
 *              paper's channel formula).  After call `epoch` every entry equals epoch * expected where
 *              expected = (M/(R*C)/Tm_p) * ceil(K/Tn_p) in WAVES and SIDE_KERNEL mode and 1 in STREAM mode; untouched
 *              in NONE.  With ag_k_chunks in effect: unsigned[R*C*k_chunks], index channel*k_chunks + chunk, expected =
 *              M/(R*C)/Tm_p (tl_query_workspace and tl_resolve report the counts).
 *   Requirements: R | M, C | M/R, R*C <= 64, Tm_p | M/(R*C), K % 8 == 0 (a last K step shorter than the kernel's is
 *   zero-filled), N % 8 == 0, Tn_p | K; violations return TL_ERR_UNSUPPORTED_SHAPE before anything is enqueued.
 *   workspace  word 0 = status word, word 1 = head of the producer-tile queue: it grows by the number of producer
 *              tiles per call, so the caller zeroes the workspace together with the flags (once, or when `epoch`
 *              restarts at 1).  Bytes 16..23 hold the start time of the call in flight when link_gbps is set.  One call at
 *              a time per workspace.  In WAVES and SIDE_KERNEL mode producer tiles are handed out through this queue to the
 *              producer workgroups and to GEMM workgroups that would otherwise wait.
 *   compute_stream receives the fused kernel; comm_stream the copies in TL_COMM_STREAM.
 */
int tl_ag_gemm(tl_ctx* ctx, const void* const* a_shards /*host array of dev*/, void* a_gathered, const void* b,
               void* c, int M, int N, int K, unsigned* flags /*dev*/, unsigned epoch, void* workspace /*dev*/,
               size_t ws_bytes, void* compute_stream, void* comm_stream);

/*
 * tl_ag_gemm for callers that cannot allocate device memory or ask anybody to: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels and bindings as tl_ag_gemm, but the
 * workspace and the channel flags live in a static device array inside the library (16.25 KiB per device, held until
 * the process ends) instead of in caller memory; this call allocates nothing.  The caller still passes inputs and outputs.
 *   - The context must have been created (tl_ctx_create sets the array up) on the device that is current at the call.
 *   - At most 4096 channel flags (R*C*k_chunks); more returns TL_ERR_WORKSPACE_TOO_SMALL before anything is enqueued.
 *   - Every call first clears the workspace and its flags on compute_stream (a fill kernel) and makes comm_stream wait
 *     for that, then runs as call number 1: no epoch to keep.  All calls on one device share the one array, so calls
 *     that overlap on a device race (also with tl_check_status); serialise them, e.g. on one pair of streams.
 *   - tl_check_status(ctx, NULL) reads and clears this array's status word (after the streams were synchronised).
 * Everything else -- arguments, requirements, streams, errors -- as tl_ag_gemm.
 */
int tl_ag_gemm_static(tl_ctx* ctx, const void* const* a_shards /*host array of R device ptrs*/, void* a_gathered /*device*/,
                      const void* b /*device*/, void* c /*device*/, int M, int N, int K, void* compute_stream /*hipStream_t*/,
                      void* comm_stream /*hipStream_t*/);

/* The first half of the MLP layer with its activation folded into the GEMM's epilogue (paper, evaluation, "MLP
 * Layer": AllGather + GEMM, then an activation layer such as SiLUMul or GeLUMul, then GEMM + ReduceScatter):
 *   Y = act(A_gathered . W_gate) * (A_gathered . W_up),   SiLUMul: act(g) = g / (1 + exp(-g));  GeLUMul: act(g) =
 *   g * Phi(g) with the exact normal distribution function; applied to the unrounded fp32 accumulators, rounded once.
 * b_gate_up [K, 2F] row-major (device) holds both projections side by side in blocks of 32 columns: column 64t + j is
 * gate feature 32t + j for j < 32 and up feature 32t + j - 32 for 32 <= j < 64 (the two values of a feature then sit
 * in one lane's accumulators).  y [M, F] row-major (device).  F % 32 == 0.  Everything else -- shards, gathered buffer,
 * flags, epochs, workspace, streams, bindings, errors -- as tl_ag_gemm with N = 2F (tl_query_workspace, tl_resolve and
 * tl_dump_schedule with dims {M, 2F, K}); the 224-wide compute tile is not available. */
enum { TL_ACT_SILU_MUL = 1, TL_ACT_GELU_MUL = 2 };
int tl_ag_gemm_act_mul(tl_ctx* ctx, const void* const* a_shards /*host array of R device ptrs*/, void* a_gathered /*device*/,
                       const void* b_gate_up /*device*/, void* y /*device*/, int M, int F, int K, int act,
                       unsigned* flags /*device*/, unsigned epoch, void* workspace /*device*/, size_t ws_bytes,
                       void* compute_stream /*hipStream_t*/, void* comm_stream /*hipStream_t*/);

/*
 * AllGather + GEMM in push mode (paper: "Data Primitives", push mode; tile_push_data + peer_tile_notify).  Everything tl_ag_gemm does, and
 * the producer side also pushes every producer tile of the LOCAL shard a_shards[r] into each peer's copy of the
 * gathered matrix and raises that peer's channel counter.  On this one-GPU stand-in the shards of the peers still
 * arrive through the library's own copies (they stand for what the peers push); those tiles head the ticket queue, the
 * pushes of the local shard follow.
 *   peer_slots  host array of R dev pointers; entry q != r is the place of this rank's shard in peer q's gathered
 *               matrix, [M/R, K] bf16 (written: an exact copy of a_shards[r]); entry r ignored.
 *   flags       dev unsigned[R*C + R*C]: the channel flags of tl_ag_gemm, then the pushed counters, index q*C + c =
 *               this rank's channel c delivered to peer q; each grows per call by the producer tiles of a channel
 *               (`expected_per_channel` of tl_resolve); entries of q = r stay untouched.
 *   comm_mode TL_COMM_WAVES or TL_COMM_SIDE_KERNEL; ag_k_chunks and link_gbps must be off.  A workspace serves one
 *   entry point and shape (the ticket counter grows by the call's number of tickets).  All else as tl_ag_gemm.
 */
int tl_ag_gemm_push(tl_ctx* ctx, const void* const* a_shards /*host array of R device ptrs*/, void* a_gathered /*device*/,
                    void* const* peer_slots /*host array of R device ptrs*/, const void* b /*device*/, void* c /*device*/, int M, int N,
                    int K, unsigned* flags /*device*/, unsigned epoch, void* workspace /*device*/, size_t ws_bytes,
                    void* compute_stream /*hipStream_t*/, void* comm_stream /*hipStream_t*/);

/*
 * GEMM + ReduceScatter (paper: "Kernel Design", GEMM + ReduceScatter; evaluation: scatter by
 * copy, reduction on compute cores).  partial[M,N] = bf16(A[M,K] . B[K,N]) is stored locally and each
 * GEMM tile notifies the reduce tiles it covers.  A reduce tile whose rows lie in this rank's segment
 * [r*M/R, (r+1)*M/R) waits for every peer, sums the R bf16 inputs in fp32 (rank order) and stores bf16
 * to `out`; a reduce tile of segment q != r is pushed into peer_push[q] and peer q is notified.
 *   peer_recv  host array of R dev pointers; entry q != r is what peer q pushed to this rank, [M/R, N] bf16
 *              (seeded by the caller); entry r ignored.
 *   peer_push  host array of R dev pointers; entry q != r is the landing zone of this rank's partial rows of
 *              segment q, [M/R, N] bf16 (written); entry r ignored.
 *   out        dev [M/R, N] bf16 (written).
 *   flags      dev unsigned[n_flags] from tl_query_workspace: first the reduce-tile ready counters
 *              (row-major over reduce tiles; +1 per covering GEMM tile), then R*(reduce tiles per segment)
 *              peer-arrival counters (peer-major; entry for peer q counts q's pushes into this rank, raised by
 *              the library's simulated peers), then the same number of pushed counters (this rank's pushes
 *              into peer q).  Each grows by its expected count per call.
 *   With tl_config.rs_direct_push the GEMM epilogue stores each output row at its final place (own segment: `partial`,
 *   segment q: peer_push[q]).  A reduce tile of another segment that one GEMM tile fills alone is then announced to its
 *   owner by that GEMM tile (its pushed counter moves together with its ready counter); reduce tiles that several GEMM
 *   tiles share are announced by the reduce side once all of them have stored their part.
 *   workspace  dev, tl_query_workspace bytes: word 0 = status word, word 1 = head of the reduce side's work queue when the
 *              reduce side is a kernel of its own (TL_COMM_SIDE_KERNEL, TL_COMM_STREAM): it grows by the number of work
 *              items per call, so the caller zeroes the workspace together with the flags (once, or when `epoch`
 *              restarts at 1), keeps `epoch` counting call by call, and runs one call at a time per workspace.
 *   Requirements: R | M, reduce tile Tm_r | M/R and Tn_r | N, K % 8 == 0, N % 8 == 0.
 */
int tl_gemm_rs(tl_ctx* ctx, const void* a, const void* b, void* partial, const void* const* peer_recv /*host array of dev*/,
               void* const* peer_push /*host array of dev*/, void* out, int M, int N, int K, unsigned* flags /*dev*/,
               unsigned epoch, void* workspace /*dev*/, size_t ws_bytes, void* compute_stream, void* comm_stream);

/*
 * GEMM + ring ReduceScatter (paper: "Kernel Design", the GEMM + ring ReduceScatter kernel: local reduction, pass the
 * partial result to the previous rank, peer_tile_wait / peer_tile_notify between neighbours).  The running sum of
 * segment q travels rank q-1 -> q-2 -> ... -> q (indices mod R); it is bf16 on every hop.  This rank r
 *   - starts the chain of segment r+1: its partial rows of that segment go to ring_push[r+1] unchanged,
 *   - for every other segment q != r: ring_push[q] = bf16(partial rows + ring_recv[q]) (fp32 sum),
 *   - ends the chain of its own segment: out = bf16(partial rows + ring_recv[r]).
 * The GEMM and the reduce side take the segments in chain order r+1, r+2, ..., r (unless tile_order is NATURAL).
 *   ring_recv  host array of R dev pointers; entry q != r+1 is the running sum of segment q that rank r+1 handed on,
 *              [M/R, N] bf16 (seeded by the caller); entry r+1 ignored.
 *   ring_push  host array of R dev pointers; entry q != r is the landing zone at rank r-1 for this rank's running sum
 *              of segment q, [M/R, N] bf16 (written); entry r ignored.
 *   flags, workspace, partial, out, requirements and error behaviour as tl_gemm_rs (sizes from tl_query_workspace with
 *   TL_OP_GEMM_RS); the arrival counters are indexed by segment (raised by the library's simulated next rank for every
 *   segment but r+1), the pushed counters by segment (every segment but r).  tl_config.rs_direct_push is ignored:
 *   every segment passes through the reduce side.
 */
int tl_gemm_ring_rs(tl_ctx* ctx, const void* a, const void* b, void* partial, const void* const* ring_recv /*host array of dev*/,
                    void* const* ring_push /*host array of dev*/, void* out, int M, int N, int K, unsigned* flags /*dev*/,
                    unsigned epoch, void* workspace /*dev*/, size_t ws_bytes, void* compute_stream, void* comm_stream);

/*
 * MoE routing -> dynamic mapping tables (paper: "Tile-Centric Mapping", dynamic mapping: the lookup tables f_S_low,
 * f_S_high, f_R, f_C, which this call fills at run time from the routing).  Enqueued on `stream`.
 *   gate_logits dev [T,E] fp32.  Per token the `topk` experts with the largest logits are taken (equal logits: the
 *               lower expert index first; listed by descending logit); weight = softmax over all E experts,
 *               divided by the sum over the selected ones if `renormalize`.
 *   topk_ids    dev [T,topk] int (written)      topk_w dev [T,topk] fp32 (written)
 *   Routed row (t,j) has id t*topk+j.  Rows are sorted by expert, ascending id inside an expert (stable):
 *   expert_offsets dev [E+1] int (written), sorted_row dev [T*topk] int (written).
 *   tile_tables dev [max_row_tiles, 8] int (written): expert e owns ceil(count[e]/tile_m) row tiles over its run of
 *               sorted rows, the last one short; one record per tile, experts ascending:
 *               f_S_low, f_S_high, expert, chan_mask_lo, chan_mask_hi, f_R_lo, f_R_hi, 0
 *               chan_mask bit (rank*C + local channel) = AllGather channel holding a token of the tile;
 *               f_R_lo..f_R_hi = span of source ranks.   n_tiles dev int[1] (written).
 *   tile_m      row-tile height; use info[0] of tl_moe_query; max_row_tiles = info[2].
 *   Requirements: E <= 64, topk <= 8, topk <= E, R | T, C | T/R, R*C <= 64.
 */
int tl_moe_route(tl_ctx* ctx, const float* gate_logits /*dev*/, int T, int E, int topk, int renormalize, int tile_m,
                 int* topk_ids /*dev*/, float* topk_w /*dev*/, int* expert_offsets /*dev*/, int* sorted_row /*dev*/,
                 int* tile_tables /*dev*/, int* n_tiles /*dev*/, void* stream);

/* Geometry of a MoE half (op = TL_OP_MOE_AG_GATHER_GEMM or TL_OP_MOE_GEMM_SCATTER_RS), host call:
 * info[0..7] = tile_m, tile_n, max_row_tiles, n_flags, workspace bytes, expected notifications per AllGather channel
 *              (part 1), tokens per top-k reduce tile (part 2), column blocks. */
int tl_moe_query(const tl_ctx* ctx, int op, int T, int H, int I, int E, int topk, int* info /*host, 8 ints*/);

/*
 * MoE part 1: AllGather + Gather + GroupGEMM (paper: "Kernel Design", AG + MoE; evaluation, MoE layer).
 * Y1[s,:] = bf16( X[sorted_row[s]/topk, :] . W1[expert(s)] ) for every sorted row s; X = AllGather of the token shards.
 * A grouped-GEMM tile waits (consumer_tile_wait through the table's channel mask) for exactly the AllGather channels
 * that hold its tokens, and loads its A rows by index.
 *   x_shards host array of R dev pointers, each [T/R,H] bf16;  x_gathered dev [T,H] bf16 (written)
 *   w1 dev [E,H,I] bf16;  sorted_row / tile_tables / n_tiles: device outputs of tl_moe_route (same tile_m)
 *   y1 dev [T*topk, I] bf16 in sorted row order (written)
 *   flags dev unsigned[R*C], workspace as for tl_ag_gemm.  comm_mode: NONE, WAVES or SIDE_KERNEL.
 *   Requirements: those of tl_moe_route, H % 64 == 0, I % 64 == 0.
 */
int tl_moe_ag_gather_gemm(tl_ctx* ctx, const void* const* x_shards /*host array of dev*/, void* x_gathered, const void* w1,
                          const int* sorted_row, const int* tile_tables, const int* n_tiles, void* y1, int T, int H, int I, int E,
                          int topk, unsigned* flags /*dev*/, unsigned epoch, void* workspace /*dev*/, size_t ws_bytes,
                          void* compute_stream, void* comm_stream);

/* MoE part 1 with the expert FFN's activation folded into the grouped GEMM's epilogue (as tl_ag_gemm_act_mul does for the
 * dense layer): Y1[s,:] = act(x . Wgate[e]) * (x . Wup[e]) for x = the token of sorted row s and e = its expert.
 * w1_gate_up dev [E, H, 2F] bf16: per expert the [H, 2F] layout of tl_ag_gemm_act_mul (32 gate columns, then the same
 * 32 up columns).  y1 dev [T*topk, F].  F % 32 == 0; tl_moe_query with I = 2F gives the geometry.  Everything else as
 * tl_moe_ag_gather_gemm; the 224-wide tile is not available. */
int tl_moe_ag_gather_gemm_act_mul(tl_ctx* ctx, const void* const* x_shards /*host array of dev*/, void* x_gathered /*dev*/,
                                  const void* w1_gate_up /*dev*/, const int* sorted_row /*dev*/, const int* tile_tables /*dev*/,
                                  const int* n_tiles /*dev*/, void* y1 /*dev*/, int T, int H, int F, int E, int topk, int act,
                                  unsigned* flags /*dev*/, unsigned epoch, void* workspace /*dev*/, size_t ws_bytes,
                                  void* compute_stream, void* comm_stream);

/*
 * MoE part 2: GroupGEMM + Scatter + TopkReduce + ReduceScatter (paper: evaluation, MoE layer: three overlapped kernels).
 *   stage A  Z[s,:] = bf16( topk_w[row] * (X2[s,:] . W2[expert(s)]) ) stored at scatter_buf[row,:], row = sorted_row[s]
 *   stage B  partial[t,:] = bf16( sum_j scatter_buf[t*topk+j,:] )            (fp32 sum)
 *   stage C  ReduceScatter of partial over ranks as in tl_gemm_rs (own segment reduced into `out`, others pushed)
 * Each stage notifies the next per tile: A -> B through per (token block, column block) row counters, B -> C per reduce tile.
 *   x2 dev [T*topk, I] bf16 sorted row order; w2 dev [E,I,H] bf16; topk_w dev [T,topk] fp32
 *   scatter_buf dev [T*topk,H] bf16 (written); partial dev [T,H] bf16 (written)
 *   peer_recv / peer_push host arrays of R dev pointers, each [T/R,H] bf16; out dev [T/R,H] bf16 (written)
 *   flags dev unsigned[info[3] of tl_moe_query]: row counters | reduce-tile ready | peer arrived | pushed
 *   With tl_config.rs_direct_push stage B stores the token blocks of another rank's segment straight into peer_push[]
 *   (and those of the own segment into `partial`) and announces them to their owner itself; stage C reduces the own segment.
 *   workspace as for tl_gemm_rs (word 1 = the work queue of stage C in TL_COMM_SIDE_KERNEL mode: zeroed with the flags).
 *   Requirements: those of tl_moe_route, H % tile_n == 0, tokens per reduce tile | T/R.  comm_mode: NONE (stage A only),
 *   WAVES or SIDE_KERNEL.
 */
int tl_moe_gemm_scatter_rs(tl_ctx* ctx, const void* x2, const void* w2, const int* sorted_row, const int* tile_tables,
                           const int* n_tiles, const float* topk_w, void* scatter_buf, void* partial,
                           const void* const* peer_recv /*host array of dev*/, void* const* peer_push /*host array of dev*/, void* out,
                           int T, int H, int I, int E, int topk, unsigned* flags /*dev*/, unsigned epoch, void* workspace /*dev*/,
                           size_t ws_bytes, void* compute_stream, void* comm_stream);

/*
 * Sequence-parallel attention: AllGather of K and V overlapped with flash attention of the local queries
 * (paper: "Kernel Design", AG KV + self-attention; evaluation, sequence-parallel self-attention).
 *   O[i,hd,:] = bf16( sum_j softmax_j( scale * Q[i,hd,:] . K[j,hd,:] ) V[j,hd,:] ),  fp32 scores, statistics and accumulation,
 *   probabilities rounded to bf16 before they multiply V.  K = AllGather of the key shards along the sequence, V likewise.
 *   Local query row i sits at sequence position rank*S/R + i; with causal != 0 it attends to positions <= its own, and only
 *   the shards 0..rank are gathered and waited for (the remaining rows of k_gathered / v_gathered are not written).
 * An attention workgroup owns (head, 256 local queries) and walks the keys in blocks of 64 from position 0; the first block
 * of every AllGather channel is preceded by consumer_tile_wait on that channel's K flag and V flag.
 *   q dev [S/R, heads, head_dim] bf16;  k_shards / v_shards host arrays of R dev pointers, each [S/R, heads, head_dim] bf16
 *   k_gathered / v_gathered dev [S, heads, head_dim] bf16 (written);  o dev [S/R, heads, head_dim] bf16 (written)
 *   flags dev unsigned[2*R*C]: K channels, then V channels; channel c covers positions [c*S/(R*C), (c+1)*S/(R*C)).
 *   Zeroed once by the caller; after call number `epoch` (1, 2, ...) a gathered channel holds epoch * info[4] of tl_attn_query.
 *   workspace dev, 256 bytes, zeroed once (word 0 status, words 1 and 2 the K and V producer queues, bytes 32..47 the clock
 *             sample tl_read_clocks returns).
 *   Requirements: head_dim == 128, R | S, S/(R*C) % 64 == 0, R*C <= 64, 16-byte aligned pointers.
 *   comm_mode: NONE (k_gathered / v_gathered are taken as complete), WAVES, SIDE_KERNEL, or COPY_ENGINE: every needed
 *   shard of K, then of V, is copied on comm_stream by the runtime's copy engines (rank_copy_data: a copy kind that keeps
 *   the compute units out of it), each copy followed by a small kernel that raises the shard's C channel flags by one
 *   (rank_notify; info[4] of tl_attn_query is 1 in this mode) -- the binding of the paper's AG KV + self-attention
 *   kernel.  link_gbps must be 0 with it.  (The plain stream binding of tl_ag_gemm is not offered: the runtime's copy
 *   kernels could not become resident beside attention workgroups that hold every compute unit while waiting for them.)
 * Returns TL_OK or a negative error; waits are bounded as in tl_ag_gemm (tl_check_status).
 */
int tl_sp_ag_attention(tl_ctx* ctx, const void* q, const void* const* k_shards /*host array of dev*/,
                       const void* const* v_shards /*host array of dev*/, void* k_gathered, void* v_gathered, void* o, int S,
                       int heads, int head_dim, int causal, float scale, unsigned* flags /*dev*/, unsigned epoch,
                       void* workspace /*dev*/, size_t ws_bytes, void* compute_stream, void* comm_stream);

/* Geometry tl_sp_ag_attention resolves (host call).  info[0..7] = queries per workgroup, keys per block, n_flags, ws_bytes,
 * expected_per_channel, shards gathered, attention workgroups, communication workgroups. */
int tl_attn_query(const tl_ctx* ctx, int S, int heads, int head_dim, int causal, int* info /*host, 8 ints*/);

/*
 * Schedule dump for bit-exact checks (host call, no GPU work).  Writes int records in schedule order
 * (position p is taken by persistent workgroup p % G in its round p / G):
 *   TL_OP_AG_GEMM : 8 ints per consumer tile: tile_id, bm, bn, row_lo, row_hi, chan_lo, chan_hi, 0
 *   TL_OP_GEMM_RS : 9 ints per GEMM tile: tile_id, bm, bn, row_lo, row_hi, cm_lo, cm_hi, cn_lo, cn_hi
 *                   (inclusive ranges of reduce tiles notified), followed by 9 ints per reduce tile in the
 *                   order the reduce workgroups visit them: rs_tile_id, cm, cn, row_lo, row_hi, col_lo, col_hi,
 *                   dest_rank, expected.
 * `cap` = capacity of `out` in ints; *n = ints needed (written even when cap is too small, then
 * TL_ERR_WORKSPACE_TOO_SMALL is returned).
 */
int tl_dump_schedule(const tl_ctx* ctx, int op, const long long* dims /*host*/, int* out /*host*/, size_t cap,
                     size_t* n /*host*/);

/* The tile shape, grid sizes and flag geometry the library resolved for `dims` (host call).
 * info[0..13] = tile_m, tile_n, tile_k, compute_workgroups, comm_workgroups, comm_tile_m, comm_tile_n,
 *               n_consumer_tiles, n_comm_tiles, expected_per_channel (per flag), threads_per_workgroup, lds_bytes,
 *               group_m, k_chunks (flags per AllGather channel; 1 unless ag_k_chunks took effect). */
int tl_resolve(const tl_ctx* ctx, int op, const long long* dims /*host*/, int* info /*host, 14 ints*/);

#ifdef __cplusplus
}
#endif
#endif /* TILELINK_MI355_H */
