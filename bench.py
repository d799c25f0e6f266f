"""Benchmark of the overlapped tensor-parallel hot path on one MI355X.

One step = AllGather+GEMM on one rank's TP=8 share of MLP-5's first half (8 shards of
[1024,8192] gathered, B [8192,3584]) followed by GEMM+ReduceScatter on its second half
(A [8192,3584] x B [3584,8192], 7 peers, output [1024,8192]); inputs are synthetic, seeded and
already resident in HBM.  Prints ONE JSON line: `value` = whole-step TFLOP/s (9.62e11 flop per step over the step
time); `ops` = per operator the fused time, the GEMM alone (repeated call, and with its input rewritten before each
call), the communication side alone, and overlap efficiency = max(alone) / fused; `roofline` = the two tile kernels
against the dense bf16 MFMA peak, with measured HBM/fabric traffic per launch; `ag_gemm_links_153` = AG+GEMM with the
shards arriving over simulated 153 GB/s links; `extras` = the whole MLP layer, the MoE halves and sequence-parallel
attention; `cpu_baseline` = the CPU oracle on the same step.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # 256 CUs x 4096 flop/clk x 2.4 GHz (dense bf16 MFMA)
# HBM/fabric bytes per fused GEMM launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in
# profiles/bench_ag_gemm_gemm_rs_mlp5_tp8.md (scaled by the plain-copy calibration): mean of AG+GEMM (784 + 56 MiB, the
# tile kernel's own work: launches without communication) and GEMM+RS with direct push (672 + 128 MiB).  A measured constant, not recomputed by this script.
HBM_TRAFFIC_BYTES_PER_LAUNCH = int(0.5 * (784 + 56 + 672 + 128) * 2 ** 20)


def cpu_baseline(np, ops, w2, w3, rank):
    """The oracle as it stands, timed on the host cores on one whole step of the workload (the same arrays the GPU
    path was given): AG+GEMM of configuration 2, then GEMM+RS of configuration 3, repeated for about ten seconds; the
    fastest pass counts."""
    flop = 2.0 * w2["M"] * w2["N"] * w2["K"] + 2.0 * w3["a"].shape[0] * w3["b"].shape[1] * w3["a"].shape[1]
    best, passes = None, 0
    t_all = time.time()
    while passes < 2 or (time.time() - t_all < 10.0 and passes < 12):     # about 10 s of CPU work
        t0 = time.time()
        ops.ag_gemm(w2["a_shards"], w2["b"])
        ops.gemm_rs(w3["a"], w3["b"], w3["peer_segments"], rank)
        dt = time.time() - t0
        best = dt if best is None else min(best, dt)
        passes += 1
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": flop / best / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"one whole step (AG+GEMM 8192x3584x8192 + GEMM+RS 8192x8192x3584, 9.6e11 flop), float64 numpy, "
                      f"best of {passes} passes: {best:.1f} s ({time.time() - t_all:.1f} s in all)"}


def extras(torch, np, tl, wl, dev, up, timed, cs, ms, mode, steps, warmup, direct_push, comm_wgs=0, copy_engine=False):
    """Secondary measurements, outside the timed step: the two MoE halves (configuration 4) and sequence-parallel
    attention (configuration 5, causal, the last rank = the one with the most keys), each fused, compute alone
    (communication off, gathered inputs complete) and communication alone."""
    res = {}
    R = 8

    def triple(make, call, flop, extra=None, clocks=False, mode=mode):
        t, mhz = {}, {}
        for name, m, alone in (("compute_alone_ms", tl.TL_COMM_NONE, 0), ("comm_alone_ms", mode, 1), ("fused_ms", mode, 0)):
            st = make(m, alone)
            st["epoch"] = 0

            def fn(st=st):
                st["epoch"] += 1
                cs.wait_stream(ms)      # one call at a time per workspace
                ms.wait_stream(cs)
                call(st)
            t[name], _ = timed(fn, steps, warmup)
            if clocks and not alone:     # shader clock of the last launch's first workgroup
                cyc, ticks = tl.tl_read_clocks(st["ctx"], st["wsp"])
                mhz["shader_mhz_" + name[:-3]] = round(cyc / max(ticks, 1) * 100.0, 0)
            for ctx_, wsp_ in [(st["ctx"], st["wsp"])] + st.get("also", []):
                tl.tl_check_status(ctx_, wsp_)
                tl.tl_ctx_destroy(ctx_)
        r = {k: round(v, 4) for k, v in t.items()}
        r["tflops"] = round(flop / t["fused_ms"] / 1e9, 1)
        r["compute_alone_tflops"] = round(flop / t["compute_alone_ms"] / 1e9, 1)
        r["frac_of_peak"] = round(flop / t["fused_ms"] / 1e9 / PEAK_BF16_TFLOPS, 4)
        r["overlap_efficiency"] = round(max(t["compute_alone_ms"], t["comm_alone_ms"]) / t["fused_ms"], 4)
        r.update(mhz)
        if extra:
            r.update(extra)
        return r

    # ---------------- the whole MLP layer (MLP-5 share, rank 0): AllGather + GEMM over gate|up weights with SiLUMul in the
    # epilogue, then GEMM + ReduceScatter on its output
    M, F, H = 8192, 3584, 8192
    wg = wl.ag_gemm_gated_inputs(M, F, H, R, config_id=6)
    w3 = wl.gemm_rs_inputs(M, H, F, R, 0, config_id=3)
    shards = [up(x) for x in wg["a_shards"]]
    a_full = torch.cat(shards).clone()
    b_gu = up(tl.pack_gate_up(wg["w_gate"], wg["w_up"]))
    y = torch.zeros((M, F), dtype=torch.int16, device=dev)
    w_down = up(w3["b"])
    partial = torch.zeros((M, H), dtype=torch.int16, device=dev)
    recv = [0] + [up(w3["peer_segments"][q]) for q in range(1, R)]
    push = [0] + [torch.zeros((M // R, H), dtype=torch.int16, device=dev) for _ in range(1, R)]
    out = torch.zeros((M // R, H), dtype=torch.int16, device=dev)

    def mlp_make(m, alone):
        st = {}
        for part, op, dims in (("p1", tl.TL_OP_AG_GEMM, [M, 2 * F, H]), ("p2", tl.TL_OP_GEMM_RS, [M, H, F])):
            ctx = tl.tl_ctx_create(world_size=R, rank=0, channels_per_rank=4, comm_mode=m, tile_order=tl.TL_ORDER_OWN_FIRST, xcd_swizzle=1,
                                   spin_timeout_us=10_000_000, comm_alone=alone, rs_direct_push=direct_push, comm_workgroups=comm_wgs)
            ws, nf = tl.tl_query_workspace(ctx, op, dims)
            st[part] = dict(ctx=ctx, ws=ws, flags=torch.zeros(nf, dtype=torch.int32, device=dev), wsp=torch.zeros(ws // 4, dtype=torch.int32, device=dev))
        st["ctx"], st["wsp"] = st["p1"]["ctx"], st["p1"]["wsp"]
        st["also"] = [(st["p2"]["ctx"], st["p2"]["wsp"])]
        st["xg"] = a_full.clone() if m == tl.TL_COMM_NONE else torch.zeros((M, H), dtype=torch.int16, device=dev)
        torch.cuda.synchronize()
        return st

    def mlp_call(st, parts=("p1", "p2")):
        if "p1" in parts:
            p = st["p1"]
            tl.tl_ag_gemm_act_mul(p["ctx"], shards, st["xg"], b_gu, y, M, F, H, tl.TL_ACT_SILU_MUL, p["flags"], st["epoch"], p["wsp"], p["ws"], cs, ms)
        if "p2" in parts:
            p = st["p2"]
            if "p1" in parts:
                ms.wait_stream(cs)      # the reduce side of part 2 may not run ahead into part 1
            tl.tl_gemm_rs(p["ctx"], y, w_down, partial, recv, push, out, M, H, F, p["flags"], st["epoch"], p["wsp"], p["ws"], cs, ms)

    flop_mlp = 2.0 * M * (2 * F) * H + 2.0 * M * H * F
    r = triple(mlp_make, mlp_call, flop_mlp, {"workload": "MLP-5 TP=8 share, rank 0: AG + GEMM [8192,8192]x[8192,2x3584] with SiLUMul, then GEMM [8192,3584]x[3584,8192] + RS"})
    for part in ("p1", "p2"):
        st = mlp_make(mode, 0)
        st["epoch"] = 0

        def fn(st=st, part=part):
            st["epoch"] += 1
            cs.wait_stream(ms)
            ms.wait_stream(cs)
            mlp_call(st, (part,))
        r[f"{part}_fused_ms"] = round(timed(fn, steps, warmup)[0], 4)
        for q in ("p1", "p2"):
            tl.tl_check_status(st[q]["ctx"], st[q]["wsp"])
            tl.tl_ctx_destroy(st[q]["ctx"])
    res["mlp_layer"] = r

    # ---------------- GEMM + ring ReduceScatter (MLP-5 part 2 share, rank 0): every segment's running sum passes through
    # the reduce side (7 x 16 MiB received, 7 x 16 MiB passed on, the own segment finished)
    wr = wl.gemm_ring_rs_inputs(M, H, F, R, 0, config_id=7)
    a_r = up(wr["a"])
    ring_recv = [0 if t is None else up(t) for t in wr["ring_recv"]]

    def ring_make(m, alone):
        ctx = tl.tl_ctx_create(world_size=R, rank=0, channels_per_rank=1, comm_mode=m, tile_order=tl.TL_ORDER_RING, xcd_swizzle=1,
                               spin_timeout_us=10_000_000, comm_alone=alone, comm_workgroups=comm_wgs)
        ws, nf = tl.tl_query_workspace(ctx, tl.TL_OP_GEMM_RS, [M, H, F])
        st = dict(ctx=ctx, ws=ws, flags=torch.zeros(nf, dtype=torch.int32, device=dev), wsp=torch.zeros(ws // 4, dtype=torch.int32, device=dev))
        torch.cuda.synchronize()
        return st

    def ring_call(st):
        tl.tl_gemm_ring_rs(st["ctx"], a_r, w_down, partial, ring_recv, push, out, M, H, F, st["flags"], st["epoch"], st["wsp"], st["ws"], cs, ms)

    # ---------------- AllGather + GEMM in push mode (MLP-5 part 1 share, rank 0): the local shard also goes to seven peers
    N1 = F
    wp = wl.ag_gemm_inputs(M, N1, H, R, config_id=2)
    p_shards = [up(x) for x in wp["a_shards"]]
    p_full = torch.cat(p_shards).clone()
    p_b, p_c = up(wp["b"]), torch.zeros((M, N1), dtype=torch.int16, device=dev)
    p_slots = [0] + [torch.zeros((M // R, H), dtype=torch.int16, device=dev) for _ in range(1, R)]

    def push_make(m, alone):
        ctx = tl.tl_ctx_create(world_size=R, rank=0, channels_per_rank=4, comm_mode=m, tile_order=tl.TL_ORDER_OWN_FIRST, xcd_swizzle=1,
                               spin_timeout_us=10_000_000, comm_alone=alone, comm_workgroups=comm_wgs)
        ws, nf = tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [M, N1, H])
        st = dict(ctx=ctx, ws=ws, flags=torch.zeros(2 * nf, dtype=torch.int32, device=dev), wsp=torch.zeros(ws // 4, dtype=torch.int32, device=dev))
        st["g"] = p_full if m == tl.TL_COMM_NONE else torch.zeros((M, H), dtype=torch.int16, device=dev)
        torch.cuda.synchronize()
        return st

    def push_call(st):
        if st["g"] is p_full:       # no communication: the plain entry point on the complete matrix
            tl.tl_ag_gemm(st["ctx"], p_shards, st["g"], p_b, p_c, M, N1, H, st["flags"], st["epoch"], st["wsp"], st["ws"], cs, ms)
        else:
            tl.tl_ag_gemm_push(st["ctx"], p_shards, st["g"], p_slots, p_b, p_c, M, N1, H, st["flags"], st["epoch"], st["wsp"], st["ws"], cs, ms)

    res["ag_gemm_push"] = triple(push_make, push_call, 2.0 * M * N1 * H,
                                 {"workload": "MLP-5 part 1 TP=8 share in push mode, rank 0: the 7 remote shards arrive (library copies standing for "
                                              "the peers' pushes) and the local shard is pushed into 7 peer slots: twice the copy traffic of the pull form"})
    del p_shards, p_full, p_b, p_c, p_slots

    res["gemm_ring_rs"] = triple(ring_make, ring_call, 2.0 * M * H * F,
                                 {"workload": "MLP-5 part 2 TP=8 share as a ring, rank 0: GEMM [8192,3584]x[3584,8192], running sums of 7 segments "
                                              "received and passed on, own segment finished"})
    del shards, a_full, b_gu, y, w_down, partial, recv, push, out, a_r, ring_recv

    # ---------------- MoE (configuration 4), rank 0
    c = wl.CONFIGS[4]
    T, H, I, E, k = c["T"], c["H"], c["I"], c["E"], c["topk"]
    w = wl.moe_inputs(T, H, I, E, k, R, 0, config_id=4)
    x_shards = [up(x) for x in w["x_shards"]]
    x_full = torch.cat(x_shards).clone()
    w1, w2, x2 = up(w["w1"].reshape(E * H, I)), up(w["w2"].reshape(E * I, H)), up(w["x2"])
    logits = torch.from_numpy(w["logits"]).to(dev)
    y1 = torch.zeros((T * k, I), dtype=torch.int16, device=dev)
    scatter = torch.zeros((T * k, H), dtype=torch.int16, device=dev)
    partial = torch.zeros((T, H), dtype=torch.int16, device=dev)
    recv = [0] + [up(w["peer_segments"][q]) for q in range(1, R)]
    push = [0] + [torch.zeros((T // R, H), dtype=torch.int16, device=dev) for _ in range(1, R)]
    out = torch.zeros((T // R, H), dtype=torch.int16, device=dev)

    def moe_state(op, m, alone, C, cols=None):
        ctx = tl.tl_ctx_create(world_size=R, rank=0, channels_per_rank=C, comm_mode=m, tile_order=tl.TL_ORDER_OWN_FIRST, xcd_swizzle=1,
                               spin_timeout_us=10_000_000, comm_alone=alone, rs_direct_push=direct_push, comm_workgroups=comm_wgs)
        q = tl.tl_moe_query(ctx, op, T, H, cols or I, E, k)
        st = dict(ctx=ctx, q=q,
                  ids=torch.zeros((T, k), dtype=torch.int32, device=dev), tw=torch.zeros((T, k), dtype=torch.float32, device=dev),
                  off=torch.zeros(E + 1, dtype=torch.int32, device=dev), srow=torch.zeros(T * k, dtype=torch.int32, device=dev),
                  tab=torch.zeros((q["max_row_tiles"], 8), dtype=torch.int32, device=dev), nt=torch.zeros(1, dtype=torch.int32, device=dev),
                  flags=torch.zeros(q["n_flags"], dtype=torch.int32, device=dev), wsp=torch.zeros(q["ws_bytes"] // 4, dtype=torch.int32, device=dev))
        with torch.cuda.stream(cs):
            tl.tl_moe_route(ctx, logits, T, E, k, True, q["tile_m"], st["ids"], st["tw"], st["off"], st["srow"], st["tab"], st["nt"])
        torch.cuda.synchronize()
        return st

    def p1_make(m, alone):
        st = moe_state(tl.TL_OP_MOE_AG_GATHER_GEMM, m, alone, 4)
        st["xg"] = x_full.clone() if m == tl.TL_COMM_NONE else torch.zeros((T, H), dtype=torch.int16, device=dev)
        return st

    def p1_call(st):
        tl.tl_moe_ag_gather_gemm(st["ctx"], x_shards, st["xg"], w1, st["srow"], st["tab"], st["nt"], y1, T, H, I, E, k, st["flags"], st["epoch"],
                                 st["wsp"], st["q"]["ws_bytes"], cs, ms)

    def p2_call(st):
        tl.tl_moe_gemm_scatter_rs(st["ctx"], x2, w2, st["srow"], st["tab"], st["nt"], st["tw"], scatter, partial, recv, push, out, T, H, I, E, k,
                                  st["flags"], st["epoch"], st["wsp"], st["q"]["ws_bytes"], cs, ms)

    flop_moe = 2.0 * T * k * H * I
    res["moe_ag_gather_gemm"] = triple(p1_make, p1_call, flop_moe, {"workload": f"T={T} H={H} I={I} E={E} top{k}, TP=8 share, rank 0"})
    res["moe_gemm_scatter_rs"] = triple(lambda m, alone: moe_state(tl.TL_OP_MOE_GEMM_SCATTER_RS, m, alone, 1), p2_call, flop_moe,
                                        {"workload": f"T={T} H={H} I={I} E={E} top{k}, TP=8 share, rank 0; compute alone = grouped GEMM + scatter only"})

    # the whole MoE layer: gather + grouped GEMM over gate|up expert weights with SiLUMul in the epilogue (I features each),
    # then grouped GEMM + scatter + top-k reduce + ReduceScatter on its output
    w1_gu = up(tl.pack_gate_up(w["w1"].reshape(E * H, I), w["w1_up"].reshape(E * H, I)))

    def layer_make(m, alone):
        p1 = moe_state(tl.TL_OP_MOE_AG_GATHER_GEMM, m, alone, 4, cols=2 * I)
        p2 = moe_state(tl.TL_OP_MOE_GEMM_SCATTER_RS, m, alone, 1)
        p1["xg"] = x_full.clone() if m == tl.TL_COMM_NONE else torch.zeros((T, H), dtype=torch.int16, device=dev)
        return dict(p1=p1, p2=p2, ctx=p1["ctx"], wsp=p1["wsp"], also=[(p2["ctx"], p2["wsp"])])

    def layer_call(st):
        p = st["p1"]
        tl.tl_moe_ag_gather_gemm_act_mul(p["ctx"], x_shards, p["xg"], w1_gu, p["srow"], p["tab"], p["nt"], y1, T, H, I, E, k, tl.TL_ACT_SILU_MUL,
                                         p["flags"], st["epoch"], p["wsp"], p["q"]["ws_bytes"], cs, ms)
        ms.wait_stream(cs)      # the reduce side of part 2 may not run ahead into part 1
        p = st["p2"]
        tl.tl_moe_gemm_scatter_rs(p["ctx"], y1, w2, p["srow"], p["tab"], p["nt"], p["tw"], scatter, partial, recv, push, out, T, H, I, E, k,
                                  p["flags"], st["epoch"], p["wsp"], p["q"]["ws_bytes"], cs, ms)

    res["moe_layer"] = triple(layer_make, layer_call, 3 * flop_moe,
                              {"workload": f"T={T} H={H} I={I} E={E} top{k}, TP=8 share, rank 0: gather + grouped GEMM [.,{H}]x[{H},2x{I}] with "
                                           f"SiLUMul, then grouped GEMM [.,{I}]x[{I},{H}] + scatter + top-k reduce + RS"})
    del x_shards, x_full, w1, w1_gu, w2, x2, y1, scatter, partial, recv, push, out

    # ---------------- sequence-parallel attention (configuration 5), causal, rank 7
    c = wl.CONFIGS[5]
    S, Hd, D, rank = c["S"], c["heads"], c["head_dim"], R - 1
    w = wl.sp_attention_inputs(S, Hd, D, R)
    S_loc = S // R
    q_dev = up(w["q_shards"][rank])
    ks, vs = [up(x) for x in w["k_shards"]], [up(x) for x in w["v_shards"]]
    k_full, v_full = torch.cat(ks).clone(), torch.cat(vs).clone()
    o = torch.zeros((S_loc, Hd, D), dtype=torch.int16, device=dev)

    def at_make(m, alone):
        ctx = tl.tl_ctx_create(world_size=R, rank=rank, channels_per_rank=1, comm_mode=m, spin_timeout_us=10_000_000, comm_alone=alone,
                               comm_workgroups=comm_wgs)
        info = tl.tl_attn_query(ctx, S, Hd, D, True)
        full = m == tl.TL_COMM_NONE
        st = dict(ctx=ctx, info=info, kg=k_full if full else torch.zeros_like(k_full), vg=v_full if full else torch.zeros_like(v_full),
                  flags=torch.zeros(info["n_flags"], dtype=torch.int32, device=dev), wsp=torch.zeros(info["ws_bytes"] // 4, dtype=torch.int32, device=dev))
        torch.cuda.synchronize()    # the fills ran on the default stream, the calls use cs and ms
        return st

    def at_call(st):
        tl.tl_sp_ag_attention(st["ctx"], q_dev, ks, vs, st["kg"], st["vg"], o, S, Hd, D, True, D ** -0.5, st["flags"], st["epoch"], st["wsp"],
                              st["info"]["ws_bytes"], cs, ms)

    g = rank * S_loc + np.arange(S_loc, dtype=np.float64)
    flop_attn = 4.0 * D * Hd * float((g + 1).sum())     # QK^T and PV over the keys a causal query sees
    res["sp_ag_attention"] = triple(at_make, at_call, flop_attn,
                                    {"workload": f"S={S} heads={Hd} head_dim={D} causal, TP=8 share, rank {rank} (keys 0..{S - 1})",
                                     "flop_count": "4*D*heads*sum_i(position_i+1): masked pairs are not counted"}, clocks=True)
    # the same with K and V gathered by the copy engines (the binding of the paper's AG-KV + attention kernel; with
    # --comm-mode copy_engine only: a profiler that serialises kernels would hold the notify kernels back behind the
    # attention kernel that waits for them).  On one GPU copying onto itself the engines move ~0.5 TB/s, so this measures
    # the binding, not what links would deliver
    if copy_engine:
        res["sp_ag_attention_copy_engine"] = triple(at_make, at_call, flop_attn,
                                                    {"workload": "as sp_ag_attention, K/V shards copied by hipMemcpyAsync(..., hipMemcpyDeviceToDeviceNoCU) "
                                                                 "on the communication stream + a notify kernel per shard"}, mode=tl.TL_COMM_COPY_ENGINE)
    return res


MLP_TABLE = {"MLP-1": (8192, 4096, 11008), "MLP-2": (8192, 4096, 14336), "MLP-3": (8192, 3584, 14336), "MLP-4": (8192, 4608, 36864),
             "MLP-5": (8192, 8192, 28672), "MLP-6": (8192, 8192, 29568)}
MOE_TABLE = {"MoE-1": (8192, 2048, 1536, 8, 2), "MoE-2": (8192, 2048, 1536, 32, 2), "MoE-3": (8192, 2048, 1536, 32, 5),
             "MoE-4": (8192, 4096, 2048, 8, 2), "MoE-5": (8192, 4096, 2048, 32, 2), "MoE-6": (8192, 4096, 2048, 32, 5)}
ATTN_TABLE = {"Attn-1": 32, "Attn-2": 64}


def shape_table(torch, tl, dev, timed, cs, ms, mode, steps, warmup, over_ag=None, over_rs=None, only=""):
    """The shapes of the paper's benchmark table (evaluation: "Benchmark Shapes"), one rank's TP=8 share each: fused,
    compute alone and communication alone per operator.  Timing only: the tensors are drawn on the GPU (N(0,1)
    activations, N(0,0.02) weights, matched peers) -- parity at these shapes is the tests' business.  The K of a
    GEMM + ReduceScatter share is rounded down to the tile kernels' K step (I/8 = 1376 -> 1344, 3696 -> 3648)."""
    R = 8
    torch.manual_seed(20313)

    def rnd(shape, std=1.0):
        return (torch.randn(shape, device=dev, dtype=torch.float32) * std).to(torch.bfloat16).view(torch.int16)

    def zeros(shape):
        return torch.zeros(shape, dtype=torch.int16, device=dev)

    def run3(make, call, flop):
        t = {}
        for name, m, alone in (("compute_alone_ms", tl.TL_COMM_NONE, 0), ("comm_alone_ms", mode, 1), ("fused_ms", mode, 0)):
            st = make(m, alone)
            st["epoch"] = 0

            def fn(st=st):
                st["epoch"] += 1
                cs.wait_stream(ms)      # one call at a time per workspace
                ms.wait_stream(cs)
                call(st)
            t[name] = timed(fn, steps, warmup)[0]
            tl.tl_check_status(st["ctx"], st["wsp"])
            tl.tl_ctx_destroy(st["ctx"])
        r = {k: round(v, 4) for k, v in t.items()}
        r["tflops"] = round(flop / t["fused_ms"] / 1e9, 1)
        r["overlap_efficiency"] = round(max(t["compute_alone_ms"], t["comm_alone_ms"]) / t["fused_ms"], 4)
        return r

    def dense_ctx(m, alone, op, dims, C):
        over = dict((over_ag if op == tl.TL_OP_AG_GEMM else over_rs) or {})
        if callable(over.get("ag_k_chunks")):
            over["ag_k_chunks"] = over["ag_k_chunks"](dims)
        ctx = tl.tl_ctx_create(world_size=R, rank=0, channels_per_rank=C, comm_mode=m, tile_order=tl.TL_ORDER_OWN_FIRST, xcd_swizzle=1,
                               spin_timeout_us=10_000_000, comm_alone=alone, rs_direct_push=1,
                               **{k: v for k, v in over.items() if m != tl.TL_COMM_NONE or k in ("tile_m", "tile_n")})
        ws, nf = tl.tl_query_workspace(ctx, op, dims)
        info = tl.tl_resolve(ctx, op, dims)
        st = dict(ctx=ctx, ws=ws, flags=torch.zeros(nf, dtype=torch.int32, device=dev), wsp=torch.zeros(ws // 4, dtype=torch.int32, device=dev), info=info)
        torch.cuda.synchronize()
        return st

    # some hundred milliseconds of load first: the chip's clocks settle under it
    wa, wb = torch.randn((8192, 8192), device=dev, dtype=torch.bfloat16), torch.randn((8192, 8192), device=dev, dtype=torch.bfloat16)
    for _ in range(400):
        torch.mm(wa, wb)
    torch.cuda.synchronize()
    del wa, wb
    table = {}
    for name, (S, H, I) in MLP_TABLE.items():
        if only and not name.startswith(only):
            continue
        N = I // R
        shards = [rnd((S // R, H)) for _ in range(R)]
        full = torch.cat(shards).clone()
        b, c = rnd((H, N), 0.02), zeros((S, N))

        def ag_make(m, alone):
            st = dense_ctx(m, alone, tl.TL_OP_AG_GEMM, [S, N, H], 4)
            st["g"] = full if m == tl.TL_COMM_NONE else zeros((S, H))
            return st

        def ag_call(st):
            tl.tl_ag_gemm(st["ctx"], shards, st["g"], b, c, S, N, H, st["flags"], st["epoch"], st["wsp"], st["ws"], cs, ms)
        row = {"ag_gemm": dict(run3(ag_make, ag_call, 2.0 * S * N * H), M=S, N=N, K=H)}
        del shards, full, b, c
        K = N                                            # the real K of the share (a multiple of 8; the tile zero-fills the tail of its last K step)
        a, b, partial = rnd((S, K)), rnd((K, H), 0.02), zeros((S, H))
        recv = [0] + [rnd((S // R, H), K ** 0.5 * 0.02) for _ in range(1, R)]
        push = [0] + [zeros((S // R, H)) for _ in range(1, R)]
        out = zeros((S // R, H))

        def rs_make(m, alone):
            return dense_ctx(m, alone, tl.TL_OP_GEMM_RS, [S, H, K], 1)

        def rs_call(st):
            tl.tl_gemm_rs(st["ctx"], a, b, partial, recv, push, out, S, H, K, st["flags"], st["epoch"], st["wsp"], st["ws"], cs, ms)
        row["gemm_rs"] = dict(run3(rs_make, rs_call, 2.0 * S * H * K), M=S, N=H, K=K)
        table[name] = row
        del a, b, partial, recv, push, out
        print(f"[shape-table] {name} {row}", file=sys.stderr, flush=True)

    for name, (T, H, I_full, E, k) in MOE_TABLE.items():
        if only and not name.startswith(only):
            continue
        I = I_full // R
        x_shards = [rnd((T // R, H)) for _ in range(R)]
        x_full = torch.cat(x_shards).clone()
        w1, w2, x2 = rnd((E * H, I), 0.02), rnd((E * I, H), 0.02), rnd((T * k, I))
        logits = torch.randn((T, E), device=dev, dtype=torch.float32)
        y1, scatter, partial = zeros((T * k, I)), zeros((T * k, H)), zeros((T, H))
        recv = [0] + [rnd((T // R, H), I ** 0.5 * 0.02) for _ in range(1, R)]
        push = [0] + [zeros((T // R, H)) for _ in range(1, R)]
        out = zeros((T // R, H))

        def moe_state(op, m, alone, C):
            ctx = tl.tl_ctx_create(world_size=R, rank=0, channels_per_rank=C, comm_mode=m, tile_order=tl.TL_ORDER_OWN_FIRST, xcd_swizzle=1,
                                   spin_timeout_us=10_000_000, comm_alone=alone, rs_direct_push=1)
            q = tl.tl_moe_query(ctx, op, T, H, I, E, k)
            st = dict(ctx=ctx, q=q, ids=torch.zeros((T, k), dtype=torch.int32, device=dev), tw=torch.zeros((T, k), dtype=torch.float32, device=dev),
                      off=torch.zeros(E + 1, dtype=torch.int32, device=dev), srow=torch.zeros(T * k, dtype=torch.int32, device=dev),
                      tab=torch.zeros((q["max_row_tiles"], 8), dtype=torch.int32, device=dev), nt=torch.zeros(1, dtype=torch.int32, device=dev),
                      flags=torch.zeros(q["n_flags"], dtype=torch.int32, device=dev), wsp=torch.zeros(q["ws_bytes"] // 4, dtype=torch.int32, device=dev))
            with torch.cuda.stream(cs):
                tl.tl_moe_route(ctx, logits, T, E, k, True, q["tile_m"], st["ids"], st["tw"], st["off"], st["srow"], st["tab"], st["nt"])
            torch.cuda.synchronize()
            return st

        def p1_make(m, alone):
            st = moe_state(tl.TL_OP_MOE_AG_GATHER_GEMM, m, alone, 4)
            st["xg"] = x_full if m == tl.TL_COMM_NONE else zeros((T, H))
            return st

        def p1_call(st):
            tl.tl_moe_ag_gather_gemm(st["ctx"], x_shards, st["xg"], w1, st["srow"], st["tab"], st["nt"], y1, T, H, I, E, k, st["flags"], st["epoch"],
                                     st["wsp"], st["q"]["ws_bytes"], cs, ms)

        def p2_call(st):
            tl.tl_moe_gemm_scatter_rs(st["ctx"], x2, w2, st["srow"], st["tab"], st["nt"], st["tw"], scatter, partial, recv, push, out, T, H, I, E, k,
                                      st["flags"], st["epoch"], st["wsp"], st["q"]["ws_bytes"], cs, ms)
        flop = 2.0 * T * k * H * I
        table[name] = {"moe_ag_gather_gemm": run3(p1_make, p1_call, flop),
                       "moe_gemm_scatter_rs": run3(lambda m, alone: moe_state(tl.TL_OP_MOE_GEMM_SCATTER_RS, m, alone, 1), p2_call, flop),
                       "T": T, "H": H, "I_share": I, "E": E, "topk": k}
        del x_shards, x_full, w1, w2, x2, logits, y1, scatter, partial, recv, push, out
        print(f"[shape-table] {name} {table[name]}", file=sys.stderr, flush=True)

    D, rank = 128, R - 1
    for name, heads in ATTN_TABLE.items():
        for S in (16384, 32768, 65536, 131072):
            if only and not name.startswith(only):
                continue
            S_loc = S // R
            q_dev = rnd((S_loc, heads, D))
            ks, vs = [rnd((S_loc, heads, D)) for _ in range(R)], [rnd((S_loc, heads, D)) for _ in range(R)]
            k_full, v_full = torch.cat(ks).clone(), torch.cat(vs).clone()
            o = zeros((S_loc, heads, D))

            def at_make(m, alone):
                ctx = tl.tl_ctx_create(world_size=R, rank=rank, channels_per_rank=1, comm_mode=m, spin_timeout_us=10_000_000, comm_alone=alone)
                info = tl.tl_attn_query(ctx, S, heads, D, True)
                nc = m == tl.TL_COMM_NONE
                st = dict(ctx=ctx, info=info, kg=k_full if nc else torch.zeros_like(k_full), vg=v_full if nc else torch.zeros_like(v_full),
                          flags=torch.zeros(info["n_flags"], dtype=torch.int32, device=dev), wsp=torch.zeros(info["ws_bytes"] // 4, dtype=torch.int32, device=dev))
                torch.cuda.synchronize()
                return st

            def at_call(st):
                tl.tl_sp_ag_attention(st["ctx"], q_dev, ks, vs, st["kg"], st["vg"], o, S, heads, D, True, D ** -0.5, st["flags"], st["epoch"],
                                      st["wsp"], st["info"]["ws_bytes"], cs, ms)
            lo = rank * S_loc
            flop = 4.0 * D * heads * (S_loc * lo + S_loc * (S_loc + 1) / 2.0)
            table[f"{name} S={S}"] = run3(at_make, at_call, flop)
            del q_dev, ks, vs, k_full, v_full, o
            print(f"[shape-table] {name} S={S} {table[f'{name} S={S}']}", file=sys.stderr, flush=True)
    return table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--comm-mode", default="side", choices=["waves", "side", "stream", "copy_engine"],
                    help="resource binding of the communication side; copy_engine (a DMA engine moves the AllGather's shards) applies to AG+GEMM, "
                         "GEMM+RS then uses the side kernel")
    ap.add_argument("--comm-workgroups", type=int, default=0)
    ap.add_argument("--channels", type=int, default=4)
    ap.add_argument("--ag-comm-tile-m", type=int, default=0, help="rows of an AllGather producer tile (default: the library's choice)")
    ap.add_argument("--ag-k-chunks", type=int, default=0,
                    help="chunks per AllGather channel along K, each with a flag of its own (1 = one flag per channel; 0 = this script's choice: "
                         "4 where all tiles of the GEMM fit into one round of workgroups -- every tile then starts with a wait --, else 1)")
    ap.add_argument("--link-gbps", type=int, default=0, help="simulated link rate per source rank for the AllGather (0 = unthrottled local copy; xGMI: 153)")
    ap.add_argument("--ag-order", default="own_first", choices=["own_first", "arrival"], help="tile order of AG+GEMM")
    ap.add_argument("--ag-tile", default="", help="compute tile of AG+GEMM as MxN (default: the library's choice)")
    ap.add_argument("--rs-tile", default="", help="compute tile of GEMM+RS as MxN (default: the library's choice)")
    ap.add_argument("--direct-push-mode", type=int, default=1, choices=[1, 2],
                    help="GEMM+RS: 1 = the epilogue pushes the other ranks' rows, 2 = it also reduces the own segment")
    ap.add_argument("--no-direct-push", action="store_true",
                    help="GEMM+RS: store every partial row locally and let the communication side copy the other ranks' rows "
                         "(default: the GEMM epilogue stores them straight into the peers' landing zones)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fused-only", action="store_true",
                    help="launch nothing but fused steps (clock settling included) and report their times: the run to put under "
                         "rocprofv3 --kernel-trace --stats, whose per-kernel averages then are those of the fused launches alone")
    ap.add_argument("--probes", action="store_true",
                    help="run only the issue probe (tl_issue_probe): time per slot of one MFMA plus a few vector instructions, two waves per "
                         "SIMD, zero operands (pinned clock), for every mode with and without the MFMA")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the secondary measurements (MoE halves, sequence-parallel attention); they are outside the timed step")
    ap.add_argument("--shape-table", action="store_true",
                    help="instead of the timed step: every shape of the paper's benchmark table (TP=8 share, rank 0; attention rank 7), "
                         "fused / compute alone / communication alone, as one JSON line")
    ap.add_argument("--shape-filter", default="", help="with --shape-table: only the rows whose name starts with this (MLP, MoE-3, Attn-1, ...)")
    ap.add_argument("--rs-comm-tile-m", type=int, default=0, help="with --shape-table: rows of a ReduceScatter reduce tile (default: the library's choice)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device copy (5 times): the known-size kernel against which the FETCH_SIZE / WRITE_SIZE counters are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the TP=8 layer; --gpus must be 1 "
              "(peers are seeded buffers in the same HBM, there are no collectives)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2503_20313_amd as tl
    import tl_workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.zeros_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": 1 << 30, "copy_calibration_bytes_written": 1 << 30, "launches": 5}))
        return
    if args.probes:
        ctx = tl.tl_ctx_create(world_size=1, rank=0, channels_per_rank=1)
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        sink = torch.zeros(1 + cus * 512, dtype=torch.float32, device=dev)
        clk = torch.zeros(2, dtype=torch.int64, device=dev)
        st = torch.cuda.Stream()
        names = {0: "nothing", 1: "6 v_fma_f32", 2: "2 v_exp_f32", 3: "v_cvt_pk_bf16_f32 + v_max3_f32", 4: "1 v_dot2c_f32_bf16"}
        res = {}
        for with_mfma in (1, 0):
            for m, what in names.items():
                if not with_mfma and m == 0:
                    continue
                times = []
                for rep in range(4):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(st)
                    slots = tl.tl_issue_probe(ctx, with_mfma, m, 20000, sink, clk, st)
                    e1.record(st)
                    torch.cuda.synchronize()
                    times.append(e0.elapsed_time(e1))
                cyc, ticks = clk.cpu().tolist()
                ms_ = min(times[1:])
                res[("mfma + " if with_mfma else "") + what] = {"ms": round(ms_, 4), "ns_per_slot_pair": round(ms_ * 1e6 / slots, 2),
                                                                "shader_mhz": round(cyc / max(ticks, 1) * 100.0, 0)}
        tl.tl_ctx_destroy(ctx)
        print(json.dumps({"issue_probe": res, "note": "two waves per SIMD, 160000 slots per wave; ns_per_slot_pair = launch time / slots per wave = the "
                                                      "time a SIMD spends on one slot of each of its two waves; one MFMA alone is 32 cycles"}))
        return
    mode = {"waves": tl.TL_COMM_WAVES, "side": tl.TL_COMM_SIDE_KERNEL, "stream": tl.TL_COMM_STREAM, "copy_engine": tl.TL_COMM_COPY_ENGINE}[args.comm_mode]
    STREAMED = (tl.TL_COMM_STREAM, tl.TL_COMM_COPY_ENGINE)

    def up(bits):
        return torch.from_numpy(bits.view(np.int16)).to(dev)

    R, rank = 8, 0
    # ---------------- AG+GEMM (configuration 2)
    M, N, K = 8192, 3584, 8192
    w2 = wl.ag_gemm_inputs(M, N, K, R, config_id=2)
    shards = [up(s) for s in w2["a_shards"]]
    gathered = torch.zeros((M, K), dtype=torch.int16, device=dev)
    # the local shard lives in its slot of the gathered buffer (symmetric-buffer layout): 7 remote shards are copied
    gathered[rank * (M // R):(rank + 1) * (M // R)].copy_(shards[rank])
    shards[rank] = gathered[rank * (M // R):(rank + 1) * (M // R)]
    a_full = torch.cat([up(s) for s in w2["a_shards"]])   # the complete A, source of the fresh-input rewrite
    b2 = up(w2["b"])
    c2 = torch.zeros((M, N), dtype=torch.int16, device=dev)
    # ---------------- GEMM+RS (configuration 3)
    M3, N3, K3 = 8192, 8192, 3584
    w3 = wl.gemm_rs_inputs(M3, N3, K3, R, rank, config_id=3)
    a3, b3 = up(w3["a"]), up(w3["b"])
    a3_src = a3.clone()
    partial = torch.zeros((M3, N3), dtype=torch.int16, device=dev)
    recv = [0 if q == rank else up(w3["peer_segments"][q]) for q in range(R)]
    push = [0 if q == rank else torch.zeros((M3 // R, N3), dtype=torch.int16, device=dev) for q in range(R)]
    out3 = torch.zeros((M3 // R, N3), dtype=torch.int16, device=dev)

    cs = torch.cuda.Stream()
    ms = torch.cuda.Stream()

    def pick_k_chunks(asked, dims, workgroups=256):
        """K chunks of the AllGather for a [M,N,K] GEMM: what was asked for, else 4 where one round of 256x256 tiles holds the
        whole GEMM (every tile then waits for remote rows before it can start, and starting on the first quarter of K is
        worth 6-10 %: the MLP-1..3 shares), else 1 (with more rounds chunks cost a few per cent)."""
        if asked:
            return asked
        m, n, k = dims
        one_round = -(-m // 256) * -(-n // 256) <= workgroups
        return 4 if one_round and k % 256 == 0 and k // 256 >= 8 else 1

    class Op:
        def __init__(self, op, dims, comm_mode, comm_alone=0, **over):
            tile = (args.ag_tile if op == tl.TL_OP_AG_GEMM else args.rs_tile) or "0x0"
            tm, tn = (int(v) for v in tile.split("x"))
            fields = dict(world_size=R, rank=rank, channels_per_rank=args.channels, comm_mode=comm_mode, tile_m=tm, tile_n=tn,
                          comm_tile_m=args.ag_comm_tile_m if op == tl.TL_OP_AG_GEMM else 0,
                          ag_k_chunks=pick_k_chunks(args.ag_k_chunks, dims) if op == tl.TL_OP_AG_GEMM and comm_mode not in STREAMED else 0,
                          link_gbps=args.link_gbps if op == tl.TL_OP_AG_GEMM and comm_mode not in STREAMED else 0,
                          comm_workgroups=args.comm_workgroups, xcd_swizzle=1,
                          tile_order=tl.TL_ORDER_ARRIVAL if op == tl.TL_OP_AG_GEMM and args.ag_order == "arrival" else tl.TL_ORDER_OWN_FIRST,
                          spin_timeout_us=10_000_000, comm_alone=comm_alone, rs_direct_push=0 if args.no_direct_push else args.direct_push_mode)
            fields.update(over)
            if op == tl.TL_OP_GEMM_RS and fields["comm_mode"] == tl.TL_COMM_COPY_ENGINE:
                fields["comm_mode"] = tl.TL_COMM_SIDE_KERNEL      # the reduction needs compute units
            self.ctx = tl.tl_ctx_create(**fields)
            self.op, self.dims = op, dims
            self.ws_bytes, n_flags = tl.tl_query_workspace(self.ctx, op, dims)
            self.flags = torch.zeros(n_flags, dtype=torch.int32, device=dev)
            self.wsp = torch.zeros(self.ws_bytes // 4, dtype=torch.int32, device=dev)
            self.epoch = 0
            self.info = tl.tl_resolve(self.ctx, op, dims)
            torch.cuda.synchronize()    # the zero fills ran on the default stream, the calls use cs and ms

        def __call__(self):
            self.epoch += 1
            cs.wait_stream(ms)          # one call at a time per workspace: the previous call's communication side has finished
            ms.wait_stream(cs)          # ... and the producer of this call may not run ahead into the previous call's GEMM
            if self.op == tl.TL_OP_AG_GEMM:
                tl.tl_ag_gemm(self.ctx, shards, gathered, b2, c2, M, N, K, self.flags, self.epoch, self.wsp, self.ws_bytes, cs, ms)
            else:
                tl.tl_gemm_rs(self.ctx, a3, b3, partial, recv, push, out3, M3, N3, K3, self.flags, self.epoch, self.wsp, self.ws_bytes, cs, ms)

    def timed(fn, steps, warmup):
        """Average ms per call over `steps` calls; events are recorded on the compute stream, and the
        comm stream is joined into it before the closing event."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(cs)
        for _ in range(steps):
            fn()
        cs.wait_stream(ms)
        e1.record(cs)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return e0.elapsed_time(e1) / steps, wall

    def timed_cold(fn, rewrite, steps, warmup):
        """As timed(), for a compute-only call whose input was written just before it (`rewrite`, not timed, on the
        compute stream): what the GEMM of a fused call sees, and what a layer sees whose input the previous layer
        produced.  Repeating the same call instead leaves its whole working set in the memory-side cache."""
        for _ in range(warmup):
            rewrite()
            fn()
        torch.cuda.synchronize()
        evs = []
        for _ in range(steps):
            with torch.cuda.stream(cs):
                rewrite()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(cs)
            fn()
            e1.record(cs)
            evs.append((e0, e1))
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in evs) / steps

    if args.shape_table:
        del shards, gathered, a_full, b2, c2, a3, b3, a3_src, partial, recv, push, out3
        table = shape_table(torch, tl, dev, timed, cs, ms, mode if mode not in STREAMED else tl.TL_COMM_SIDE_KERNEL, min(args.steps, 20), 3,
                            over_ag=dict(ag_k_chunks=lambda dims: pick_k_chunks(args.ag_k_chunks, dims), comm_tile_m=args.ag_comm_tile_m, comm_workgroups=args.comm_workgroups,
                                         tile_m=int((args.ag_tile or "0x0").split("x")[0]), tile_n=int((args.ag_tile or "0x0").split("x")[1])),
                            over_rs=dict(comm_tile_m=args.rs_comm_tile_m, comm_workgroups=args.comm_workgroups), only=args.shape_filter)
        print(json.dumps({"shape_table": table, "data": "synthetic", "dtype": "bf16", "n_gpus": 1}))
        return
    flop2, flop3 = 2.0 * M * N * K, 2.0 * M3 * N3 * K3
    res = {}
    ops_ = {}
    # the chip needs some hundred milliseconds of load to settle its clocks: without this the first per-operator
    # timings below (not the timed steps, which come last) read up to 15 % slow
    pre_mode = mode if args.fused_only else tl.TL_COMM_NONE
    pre = [Op(tl.TL_OP_AG_GEMM, [M, N, K], pre_mode), Op(tl.TL_OP_GEMM_RS, [M3, N3, K3], pre_mode)]
    gathered.copy_(torch.cat(shards))
    for _ in range(300):
        pre[0]()
        pre[1]()
    torch.cuda.synchronize()
    for o in pre:
        tl.tl_ctx_destroy(o.ctx)
    for name, op, dims in (("ag_gemm", tl.TL_OP_AG_GEMM, [M, N, K]), ("gemm_rs", tl.TL_OP_GEMM_RS, [M3, N3, K3])):
        fused = Op(op, dims, mode)
        if args.fused_only:
            t_fused, _ = timed(fused, args.steps, args.warmup)
            tl.tl_check_status(fused.ctx, fused.wsp)
            cyc, ticks = tl.tl_read_clocks(fused.ctx, fused.wsp)
            res[name] = {"fused_ms": round(t_fused, 4), "tflops": round((flop2 if op == tl.TL_OP_AG_GEMM else flop3) / t_fused / 1e9, 1),
                         "shader_mhz_fused": round(cyc / max(ticks, 1) * 100.0, 0), "shader_mhz_compute_alone": None,
                         "tile": f"{fused.info['tile_m']}x{fused.info['tile_n']}", "compute_workgroups": fused.info["compute_workgroups"],
                         "comm_workgroups": fused.info["comm_workgroups"]}
            ops_[name] = fused
            continue
        alone, comm = Op(op, dims, tl.TL_COMM_NONE), Op(op, dims, mode, comm_alone=1)
        if op == tl.TL_OP_AG_GEMM:
            fused()                      # leaves the gathered buffer complete for the compute-alone variant
            torch.cuda.synchronize()
        t_alone, _ = timed(alone, args.steps, args.warmup)
        if op == tl.TL_OP_AG_GEMM:
            t_cold = timed_cold(alone, lambda: gathered.copy_(a_full), args.steps, args.warmup)
        else:
            t_cold = timed_cold(alone, lambda: a3.copy_(a3_src), args.steps, args.warmup)
        t_comm, _ = timed(comm, args.steps, args.warmup)
        t_fused, _ = timed(fused, args.steps, args.warmup)
        for o in (fused, alone, comm):
            tl.tl_check_status(o.ctx, o.wsp)
        mhz = {}
        for key, o in (("fused", fused), ("compute_alone", alone)):     # shader clock of the last launch's first workgroup
            cyc, ticks = tl.tl_read_clocks(o.ctx, o.wsp)
            mhz[key] = round(cyc / max(ticks, 1) * 100.0, 0)
        fl = flop2 if op == tl.TL_OP_AG_GEMM else flop3
        res[name] = {"fused_ms": round(t_fused, 4), "compute_alone_ms": round(t_alone, 4), "comm_alone_ms": round(t_comm, 4),
                     "tflops": round(fl / t_fused / 1e9, 1), "frac_of_peak": round(fl / t_fused / 1e9 / PEAK_BF16_TFLOPS, 4),
                     "compute_alone_tflops": round(fl / t_alone / 1e9, 1),
                     "overlap_efficiency": round(max(t_alone, t_comm) / t_fused, 4),
                     "shader_mhz_fused": mhz["fused"], "shader_mhz_compute_alone": mhz["compute_alone"],
                     "compute_alone_fresh_input_ms": round(t_cold, 4),
                     "overlap_efficiency_fresh_input": round(max(t_cold, t_comm) / t_fused, 4),
                     "paper_overlap_ratio": round((t_alone + t_comm - t_fused) / t_comm, 4),
                     "tile": f"{fused.info['tile_m']}x{fused.info['tile_n']}", "compute_workgroups": fused.info["compute_workgroups"],
                     "comm_workgroups": fused.info["comm_workgroups"]}
        ops_[name] = fused

    # ---------------- the timed region proper: K steps of the whole hot path
    def step():
        ops_["ag_gemm"]()
        ops_["gemm_rs"]()

    ms_step, wall_step = timed(step, args.steps, args.warmup)
    for o in ops_.values():
        tl.tl_check_status(o.ctx, o.wsp)
    tflops = (flop2 + flop3) / ms_step / 1e9

    # ---------------- what the matrix cores alone sustain on this data: MFMA-only register loop, operands drawn like the
    # GEMM's (activations N(0,1), weights N(0,0.02)); the clock the chip grants depends on the operand values
    if args.fused_only:
        dom_ms = 0.5 * (res["ag_gemm"]["fused_ms"] + res["gemm_rs"]["fused_ms"])
        print(json.dumps({"metric": "TFLOP/s + overlap efficiency, AG+GEMM & GEMM+RS at TP=8 share, 1 MI355X", "value": round(tflops, 1),
                          "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
                          "higher_is_better": True, "dtype": "bf16", "data": "synthetic", "fused_only": True, "ops": res,
                          "roofline": {"bound": "mfma", "achieved": round(flop2 / dom_ms / 1e9, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                       "frac": round(flop2 / dom_ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                                       "kernel_ms": round(dom_ms, 4)}}))
        return
    n_thr = torch.cuda.get_device_properties(0).multi_processor_count * 512
    opnd = torch.cat([torch.randn((n_thr, 32), device=dev, dtype=torch.float32), torch.randn((n_thr, 16), device=dev, dtype=torch.float32) * 0.02],
                     dim=1).to(torch.bfloat16).contiguous()
    sink = torch.zeros(n_thr, dtype=torch.float32, device=dev)
    clk = torch.zeros(2, dtype=torch.int64, device=dev)
    pctx = ops_["ag_gemm"].ctx
    probe_iters, probe_ms, probe_flop = 20000, [], 0.0
    for i in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(cs)
        probe_flop = tl.tl_mfma_peak_probe(pctx, opnd, opnd.numel() * 2, probe_iters, sink, clk, cs)
        e1.record(cs)
        torch.cuda.synchronize()
        probe_ms.append(e0.elapsed_time(e1))
    mfma_only_tflops = probe_flop / (sum(probe_ms[2:]) / 3.0) / 1e9
    pc = clk.cpu().tolist()
    mfma_only_mhz = round(pc[0] / max(pc[1], 1) * 100.0, 0)
    del opnd, sink

    # dominant kernel = the fused GEMM kernels (AG+GEMM and GEMM+RS have the same flop count); the
    # average launch duration is the fused time measured above on the stream the kernel runs on
    dom_ms = 0.5 * (res["ag_gemm"]["fused_ms"] + res["gemm_rs"]["fused_ms"])
    achieved = flop2 / dom_ms / 1e9
    out = {
        "metric": "TFLOP/s + overlap efficiency, AG+GEMM & GEMM+RS at TP=8 share, 1 MI355X",
        "value": round(tflops, 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "MLP-5 TP=8 share: AG+GEMM 8x[1024,8192]->[8192,8192]x[8192,3584] then GEMM+RS [8192,3584]x[3584,8192]->[1024,8192]",
                   "world_size": R, "rank": rank, "comm_mode": args.comm_mode, "channels_per_rank": args.channels,
                   "rs_direct_push": 0 if args.no_direct_push else args.direct_push_mode, "ag_k_chunks": ops_["ag_gemm"].info["k_chunks"], "ag_order": args.ag_order, "link_gbps": args.link_gbps},
        "overlap_efficiency": round(min(res["ag_gemm"]["overlap_efficiency"], res["gemm_rs"]["overlap_efficiency"]), 4),
        "frac_of_bf16_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "ops": res,
        "roofline": {"bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": HBM_TRAFFIC_BYTES_PER_LAUNCH,
                     "traffic_source": "constant from the FETCH_SIZE / WRITE_SIZE counter runs in profiles/bench_ag_gemm_gemm_rs_mlp5_tp8.md, "
                                       "not measured by this run",
                     "kernel": "ag_gemm_kernel / gemm_rs_kernel (4.81e11 flop per launch each)",
                     "mfma_only_tflops": round(mfma_only_tflops, 1), "mfma_only_shader_mhz": mfma_only_mhz,
                     "frac_of_sustained": round(achieved / mfma_only_tflops, 4),
                     "shader_mhz": {k: {"fused": v["shader_mhz_fused"], "compute_alone": v["shader_mhz_compute_alone"]} for k, v in res.items()},
                     "note": "mfma_only_tflops = MFMA-only register loop (tl_mfma_peak_probe, 8 waves per compute unit) on operands drawn like the "
                             "GEMM's: what the matrix cores sustain at the clock the chip grants for this data; frac is against the datasheet peak"},
        "host_wall_ms_per_step": round(wall_step, 4),
    }
    if not args.no_extras and mode not in STREAMED:
        # AG+GEMM with the shards arriving over simulated xGMI links (153 GB/s per source rank, all side by side), arrival
        # tile order.  (Four K chunks per channel are 2 % faster still, but need the producer kernel to run beside the
        # GEMM, which a profiler that serialises kernels does not allow.)
        links = dict(link_gbps=153, tile_order=tl.TL_ORDER_ARRIVAL, ag_k_chunks=0)
        f_l, c_l = Op(tl.TL_OP_AG_GEMM, [M, N, K], mode, **links), Op(tl.TL_OP_AG_GEMM, [M, N, K], mode, comm_alone=1, **links)
        t_cl, _ = timed(c_l, args.steps, args.warmup)
        t_fl, _ = timed(f_l, args.steps, args.warmup)
        for o in (f_l, c_l):
            tl.tl_check_status(o.ctx, o.wsp)
            tl.tl_ctx_destroy(o.ctx)
        out["ag_gemm_links_153"] = {"fused_ms": round(t_fl, 4), "comm_alone_ms": round(t_cl, 4), "compute_alone_ms": res["ag_gemm"]["compute_alone_ms"],
                                    "overlap_efficiency": round(max(res["ag_gemm"]["compute_alone_ms"], t_cl) / t_fl, 4),
                                    "link_time_ms": round((M // R) * K * 2 / 153e9 * 1e3, 4), "tile_order": "arrival", "ag_k_chunks": 1}
    if not args.no_extras:
        out["extras"] = extras(torch, np, tl, wl, dev, up, timed, cs, ms, mode if mode not in STREAMED else tl.TL_COMM_SIDE_KERNEL,
                               args.steps, args.warmup, 0 if args.no_direct_push else 1, args.comm_workgroups,
                               copy_engine=mode == tl.TL_COMM_COPY_ENGINE)
    if not args.no_cpu_baseline:
        from oracle import ops as oracle_ops
        out["cpu_baseline"] = cpu_baseline(np, oracle_ops, w2, w3, rank)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
