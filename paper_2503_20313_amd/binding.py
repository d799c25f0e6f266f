"""ctypes binding of libtilelink_mi355.so: same names as the C ABI, argument marshalling only.

Device buffers are passed as torch tensors (their data_ptr() is used) or as integer
addresses.  Every function raises TileLinkError when the library returns a negative status.
There is no fallback: if the library has not been built, importing this module fails.
"""
from __future__ import annotations

import ctypes
import os

try:
    # The library must use the same HIP runtime instance as the owner of the device buffers it is given.  PyTorch ships
    # its own copy of the runtime: loading torch first makes the dynamic loader resolve this library against that copy.
    import torch  # noqa: F401
except ImportError:
    torch = None

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtilelink_mi355.so")

TL_OK, TL_ERR_INVALID_ARG, TL_ERR_UNSUPPORTED_SHAPE, TL_ERR_WORKSPACE_TOO_SMALL, TL_ERR_HIP, TL_ERR_TIMEOUT = 0, -1, -2, -3, -4, -5
TL_COMM_NONE, TL_COMM_WAVES, TL_COMM_STREAM, TL_COMM_SIDE_KERNEL, TL_COMM_EXTERNAL, TL_COMM_COPY_ENGINE = 0, 1, 2, 3, 4, 5
TL_ORDER_NATURAL, TL_ORDER_RING, TL_ORDER_OWN_FIRST, TL_ORDER_ARRIVAL = 0, 1, 2, 3
TL_ACT_SILU_MUL, TL_ACT_GELU_MUL = 1, 2
TL_OP_AG_GEMM, TL_OP_GEMM_RS, TL_OP_MOE_AG_GATHER_GEMM, TL_OP_MOE_GEMM_SCATTER_RS, TL_OP_SP_AG_ATTENTION = 0, 1, 2, 3, 4


class TileLinkError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"tilelink_mi355 status {status}: {message}")
        self.status = status


class tl_config(ctypes.Structure):
    _fields_ = [("world_size", ctypes.c_int), ("rank", ctypes.c_int), ("channels_per_rank", ctypes.c_int),
                ("tile_m", ctypes.c_int), ("tile_n", ctypes.c_int), ("comm_tile_m", ctypes.c_int),
                ("comm_tile_n", ctypes.c_int), ("comm_mode", ctypes.c_int), ("comm_workgroups", ctypes.c_int),
                ("compute_workgroups", ctypes.c_int), ("tile_order", ctypes.c_int), ("xcd_swizzle", ctypes.c_int),
                ("group_m", ctypes.c_int), ("spin_timeout_us", ctypes.c_uint), ("comm_alone", ctypes.c_int),
                ("rs_direct_push", ctypes.c_int), ("ag_k_chunks", ctypes.c_int), ("link_gbps", ctypes.c_int)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
                      "or python paper_2503_20313_amd/build.py). There is no CPU fallback.")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _i, _u, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint, ctypes.c_size_t
_lib.tl_last_error.restype = ctypes.c_char_p
_lib.tl_version.restype = ctypes.c_char_p
_lib.tl_ctx_create.argtypes = [ctypes.POINTER(tl_config), ctypes.POINTER(_vp)]
_lib.tl_ctx_create_host.argtypes = [ctypes.POINTER(tl_config), _i, ctypes.POINTER(_vp)]
_lib.tl_ctx_destroy.argtypes = [_vp]
_lib.tl_query_workspace.argtypes = [_vp, _i, ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(_sz), ctypes.POINTER(_sz)]
_lib.tl_check_status.argtypes = [_vp, _vp]
_lib.tl_read_clocks.argtypes = [_vp, _vp, ctypes.POINTER(ctypes.c_longlong)]
_lib.tl_mfma_peak_probe.argtypes = [_vp, _vp, _sz, _i, _vp, _vp, _vp, ctypes.POINTER(ctypes.c_double)]
_lib.tl_issue_probe.argtypes = [_vp, _i, _i, _i, _vp, _vp, _vp, ctypes.POINTER(ctypes.c_double)]
_lib.tl_resolve.argtypes = [_vp, _i, ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(_i)]
_lib.tl_dump_schedule.argtypes = [_vp, _i, ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(_i), _sz, ctypes.POINTER(_sz)]
_lib.tl_ag_gemm.argtypes = [_vp, ctypes.POINTER(_vp), _vp, _vp, _vp, _i, _i, _i, _vp, _u, _vp, _sz, _vp, _vp]
_lib.tl_ag_gemm_static.argtypes = [_vp, ctypes.POINTER(_vp), _vp, _vp, _vp, _i, _i, _i, _vp, _vp]
_lib.tl_ag_gemm_act_mul.argtypes = [_vp, ctypes.POINTER(_vp), _vp, _vp, _vp, _i, _i, _i, _i, _vp, _u, _vp, _sz, _vp, _vp]
_lib.tl_gemm_rs.argtypes = [_vp, _vp, _vp, _vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _vp, _i, _i, _i, _vp, _u, _vp, _sz, _vp, _vp]
_lib.tl_gemm_ring_rs.argtypes = _lib.tl_gemm_rs.argtypes
_lib.tl_ag_gemm_push.argtypes = [_vp, ctypes.POINTER(_vp), _vp, ctypes.POINTER(_vp), _vp, _vp, _i, _i, _i, _vp, _u, _vp, _sz, _vp, _vp]

_ip, _fp = ctypes.c_void_p, ctypes.c_void_p
_lib.tl_moe_query.argtypes = [_vp, _i, _i, _i, _i, _i, _i, ctypes.POINTER(_i)]
_lib.tl_moe_route.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.tl_moe_ag_gather_gemm.argtypes = [_vp, ctypes.POINTER(_vp), _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _u, _vp, _sz, _vp, _vp]
_lib.tl_moe_ag_gather_gemm_act_mul.argtypes = [_vp, ctypes.POINTER(_vp), _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _u, _vp, _sz, _vp, _vp]
_lib.tl_moe_gemm_scatter_rs.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _vp,
                                        _i, _i, _i, _i, _i, _vp, _u, _vp, _sz, _vp, _vp]
_lib.tl_sp_ag_attention.restype = _i
_lib.tl_sp_ag_attention.argtypes = [_vp, _vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _vp, _vp, _vp, _i, _i, _i, _i, ctypes.c_float, _vp, _u, _vp, _sz,
                                    _vp, _vp]
_lib.tl_attn_query.restype = _i
_lib.tl_attn_query.argtypes = [_vp, _i, _i, _i, _i, ctypes.POINTER(_i)]


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()          # torch tensor


def _ptr_array(items):
    arr = (_vp * len(items))()
    for i, it in enumerate(items):
        arr[i] = _ptr(it)
    return arr


def _stream(s):
    if s is None or isinstance(s, int):
        return s
    return s.cuda_stream         # torch.cuda.Stream


def _check(status):
    if status < 0:
        raise TileLinkError(status, _lib.tl_last_error().decode())
    return status


def _dims(dims):
    return (ctypes.c_longlong * len(dims))(*dims)


def tl_version():
    return _lib.tl_version().decode()


def tl_last_error():
    return _lib.tl_last_error().decode()


def tl_ctx_create(**fields):
    cfg = tl_config(**fields)
    ctx = _vp()
    _check(_lib.tl_ctx_create(ctypes.byref(cfg), ctypes.byref(ctx)))
    return ctx


def tl_ctx_create_host(num_compute_units=256, **fields):
    cfg = tl_config(**fields)
    ctx = _vp()
    _check(_lib.tl_ctx_create_host(ctypes.byref(cfg), num_compute_units, ctypes.byref(ctx)))
    return ctx


def tl_ctx_destroy(ctx):
    _check(_lib.tl_ctx_destroy(ctx))


def tl_query_workspace(ctx, op, dims):
    ws, nf = _sz(), _sz()
    _check(_lib.tl_query_workspace(ctx, op, _dims(dims), ctypes.byref(ws), ctypes.byref(nf)))
    return ws.value, nf.value


def tl_check_status(ctx, workspace):
    _check(_lib.tl_check_status(ctx, _ptr(workspace)))


def tl_issue_probe(ctx, with_mfma, mode, iters, sink, clocks, stream=None):
    """Enqueues the issue probe (one MFMA per slot plus the vector instructions of `mode`); returns the slots per wave."""
    slots = ctypes.c_double()
    _check(_lib.tl_issue_probe(ctx, int(with_mfma), int(mode), int(iters), _ptr(sink), _ptr(clocks), _stream(stream), ctypes.byref(slots)))
    return slots.value


def tl_read_clocks(ctx, workspace):
    """(shader cycles, 100 MHz ticks) of the last call's first compute workgroup; cycles / ticks * 100 = MHz."""
    out = (ctypes.c_longlong * 2)()
    _check(_lib.tl_read_clocks(ctx, _ptr(workspace), out))
    return int(out[0]), int(out[1])


def tl_mfma_peak_probe(ctx, operands, operand_bytes, iters, sink, clocks, stream=None):
    """Enqueues the MFMA-only loop; returns the matrix work of the launch in flop."""
    flop = ctypes.c_double()
    _check(_lib.tl_mfma_peak_probe(ctx, _ptr(operands), operand_bytes, iters, _ptr(sink), _ptr(clocks), _stream(stream), ctypes.byref(flop)))
    return flop.value


def tl_resolve(ctx, op, dims):
    info = (_i * 14)()
    _check(_lib.tl_resolve(ctx, op, _dims(dims), info))
    keys = ["tile_m", "tile_n", "tile_k", "compute_workgroups", "comm_workgroups", "comm_tile_m", "comm_tile_n",
            "n_consumer_tiles", "n_comm_tiles", "expected_per_channel", "threads_per_workgroup", "lds_bytes", "group_m",
            "k_chunks"]
    return dict(zip(keys, list(info)))


def tl_dump_schedule(ctx, op, dims):
    n = _sz()
    d = _dims(dims)
    st = _lib.tl_dump_schedule(ctx, op, d, None, 0, ctypes.byref(n))
    if st not in (TL_OK, TL_ERR_WORKSPACE_TOO_SMALL):
        _check(st)
    buf = (_i * n.value)()
    _check(_lib.tl_dump_schedule(ctx, op, d, buf, n.value, ctypes.byref(n)))
    return list(buf)


def tl_ag_gemm(ctx, a_shards, a_gathered, b, c, M, N, K, flags, epoch, workspace, ws_bytes, compute_stream=None, comm_stream=None):
    _check(_lib.tl_ag_gemm(ctx, _ptr_array(a_shards), _ptr(a_gathered), _ptr(b), _ptr(c), M, N, K, _ptr(flags), epoch,
                           _ptr(workspace), ws_bytes, _stream(compute_stream), _stream(comm_stream)))


def tl_ag_gemm_static(ctx, a_shards, a_gathered, b, c, M, N, K, compute_stream=None, comm_stream=None):
    _check(_lib.tl_ag_gemm_static(ctx, _ptr_array(a_shards), _ptr(a_gathered), _ptr(b), _ptr(c), M, N, K, _stream(compute_stream), _stream(comm_stream)))


def tl_ag_gemm_act_mul(ctx, a_shards, a_gathered, b_gate_up, y, M, F, K, act, flags, epoch, workspace, ws_bytes, compute_stream=None, comm_stream=None):
    _check(_lib.tl_ag_gemm_act_mul(ctx, _ptr_array(a_shards), _ptr(a_gathered), _ptr(b_gate_up), _ptr(y), M, F, K, act, _ptr(flags), epoch,
                                   _ptr(workspace), ws_bytes, _stream(compute_stream), _stream(comm_stream)))


def pack_gate_up(w_gate, w_up):
    """[K, F] gate and up weights (numpy arrays or torch tensors of one dtype) -> the [K, 2F] layout tl_ag_gemm_act_mul
    reads: blocks of 32 gate columns alternate with the blocks of the same 32 up columns.  F % 32 == 0."""
    K, F = w_gate.shape
    if tuple(w_up.shape) != (K, F) or F % 32:
        raise ValueError("gate and up must both be [K, F] with F a multiple of 32")
    g, u = w_gate.reshape(K, F // 32, 1, 32), w_up.reshape(K, F // 32, 1, 32)
    if torch is not None and isinstance(w_gate, torch.Tensor):
        return torch.cat([g, u], dim=2).reshape(K, 2 * F).contiguous()
    import numpy as np
    return np.ascontiguousarray(np.concatenate([g, u], axis=2).reshape(K, 2 * F))


def tl_gemm_rs(ctx, a, b, partial, peer_recv, peer_push, out, M, N, K, flags, epoch, workspace, ws_bytes, compute_stream=None, comm_stream=None):
    _check(_lib.tl_gemm_rs(ctx, _ptr(a), _ptr(b), _ptr(partial), _ptr_array(peer_recv), _ptr_array(peer_push), _ptr(out), M, N, K,
                           _ptr(flags), epoch, _ptr(workspace), ws_bytes, _stream(compute_stream), _stream(comm_stream)))


def tl_ag_gemm_push(ctx, a_shards, a_gathered, peer_slots, b, c, M, N, K, flags, epoch, workspace, ws_bytes, compute_stream=None, comm_stream=None):
    _check(_lib.tl_ag_gemm_push(ctx, _ptr_array(a_shards), _ptr(a_gathered), _ptr_array(peer_slots), _ptr(b), _ptr(c), M, N, K, _ptr(flags), epoch,
                                _ptr(workspace), ws_bytes, _stream(compute_stream), _stream(comm_stream)))


def tl_gemm_ring_rs(ctx, a, b, partial, ring_recv, ring_push, out, M, N, K, flags, epoch, workspace, ws_bytes, compute_stream=None, comm_stream=None):
    _check(_lib.tl_gemm_ring_rs(ctx, _ptr(a), _ptr(b), _ptr(partial), _ptr_array(ring_recv), _ptr_array(ring_push), _ptr(out), M, N, K,
                                _ptr(flags), epoch, _ptr(workspace), ws_bytes, _stream(compute_stream), _stream(comm_stream)))


def tl_moe_query(ctx, op, T, H, I, E, topk):
    info = (_i * 8)()
    _check(_lib.tl_moe_query(ctx, op, T, H, I, E, topk, info))
    keys = ["tile_m", "tile_n", "max_row_tiles", "n_flags", "ws_bytes", "expected_per_channel", "tokens_per_reduce_tile", "col_blocks"]
    return dict(zip(keys, list(info)))


def tl_moe_route(ctx, gate_logits, T, E, topk, renormalize, tile_m, topk_ids, topk_w, expert_offsets, sorted_row, tile_tables, n_tiles, stream=None):
    _check(_lib.tl_moe_route(ctx, _ptr(gate_logits), T, E, topk, int(renormalize), tile_m, _ptr(topk_ids), _ptr(topk_w), _ptr(expert_offsets),
                             _ptr(sorted_row), _ptr(tile_tables), _ptr(n_tiles), _stream(stream)))


def tl_moe_ag_gather_gemm_act_mul(ctx, x_shards, x_gathered, w1_gate_up, sorted_row, tile_tables, n_tiles, y1, T, H, F, E, topk, act, flags, epoch,
                                  workspace, ws_bytes, compute_stream=None, comm_stream=None):
    _check(_lib.tl_moe_ag_gather_gemm_act_mul(ctx, _ptr_array(x_shards), _ptr(x_gathered), _ptr(w1_gate_up), _ptr(sorted_row), _ptr(tile_tables),
                                              _ptr(n_tiles), _ptr(y1), T, H, F, E, topk, act, _ptr(flags), epoch, _ptr(workspace), ws_bytes,
                                              _stream(compute_stream), _stream(comm_stream)))


def tl_moe_ag_gather_gemm(ctx, x_shards, x_gathered, w1, sorted_row, tile_tables, n_tiles, y1, T, H, I, E, topk, flags, epoch, workspace, ws_bytes,
                          compute_stream=None, comm_stream=None):
    _check(_lib.tl_moe_ag_gather_gemm(ctx, _ptr_array(x_shards), _ptr(x_gathered), _ptr(w1), _ptr(sorted_row), _ptr(tile_tables), _ptr(n_tiles),
                                      _ptr(y1), T, H, I, E, topk, _ptr(flags), epoch, _ptr(workspace), ws_bytes, _stream(compute_stream),
                                      _stream(comm_stream)))


def tl_moe_gemm_scatter_rs(ctx, x2, w2, sorted_row, tile_tables, n_tiles, topk_w, scatter_buf, partial, peer_recv, peer_push, out, T, H, I, E, topk,
                           flags, epoch, workspace, ws_bytes, compute_stream=None, comm_stream=None):
    _check(_lib.tl_moe_gemm_scatter_rs(ctx, _ptr(x2), _ptr(w2), _ptr(sorted_row), _ptr(tile_tables), _ptr(n_tiles), _ptr(topk_w), _ptr(scatter_buf),
                                       _ptr(partial), _ptr_array(peer_recv), _ptr_array(peer_push), _ptr(out), T, H, I, E, topk, _ptr(flags), epoch,
                                       _ptr(workspace), ws_bytes, _stream(compute_stream), _stream(comm_stream)))


def tl_attn_query(ctx, S, heads, head_dim, causal):
    info = (_i * 8)()
    _check(_lib.tl_attn_query(ctx, S, heads, head_dim, int(causal), info))
    keys = ("block_q", "block_kv", "n_flags", "ws_bytes", "expected_per_channel", "shards_gathered", "attention_workgroups", "comm_workgroups")
    return dict(zip(keys, list(info)))


def tl_sp_ag_attention(ctx, q, k_shards, v_shards, k_gathered, v_gathered, o, S, heads, head_dim, causal, scale, flags, epoch, workspace, ws_bytes,
                       compute_stream=None, comm_stream=None):
    _check(_lib.tl_sp_ag_attention(ctx, _ptr(q), _ptr_array(k_shards), _ptr_array(v_shards), _ptr(k_gathered), _ptr(v_gathered), _ptr(o), S, heads,
                                   head_dim, int(causal), float(scale), _ptr(flags), epoch, _ptr(workspace), ws_bytes, _stream(compute_stream),
                                   _stream(comm_stream)))
