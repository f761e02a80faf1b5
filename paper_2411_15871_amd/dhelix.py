"""ctypes binding of libdhelix (include/dhelix.h): argument marshalling only.

Every function has the name of the C entry point it calls.  Tensors are passed as torch tensors
(their data_ptr is handed over) or raw integers; streams as torch.cuda.Stream, raw hipStream_t
integers or None.  Importing this module fails loudly if the library has not been built: there is
no fallback path.
"""
import ctypes as C
import os

import torch  # noqa: F401  -- first, so that libdhelix binds to the HIP runtime PyTorch has already loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdhelix.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError("libdhelix.so is not built: run `python -m paper_2411_15871_amd.build` (needs hipcc)")
lib = C.CDLL(_LIB_PATH)

DH_OK, DH_ERR_INVALID_ARG, DH_ERR_SHAPE, DH_ERR_WORKSPACE_TOO_SMALL = 0, -1, -2, -3
DH_ERR_PLAN_INVALID, DH_ERR_HIP, DH_ERR_UNSUPPORTED = -4, -5, -6
DH_F32, DH_BF16 = 0, 1
DH_ARCH_LLAMA, DH_ARCH_GPT, DH_ARCH_MOE, DH_ARCH_LLAMA_CP = 0, 1, 2, 3
DH_ROPE_HALVES, DH_ROPE_ADJACENT = 0, 1
DH_GELU_TANH, DH_GELU_ERF = 0, 1
DH_WS_FWD, DH_WS_BWD, DH_WS_SI = 0, 1, 2
DH_COMM_ALLREDUCE, DH_COMM_ALLGATHER, DH_COMM_REDUCESCATTER = 0, 1, 2
DH_COMM_A2A_DISPATCH, DH_COMM_A2A_COMBINE = 3, 4
DH_MAX_OPS, DH_MAX_DEPS = 32, 96


def op_names(arch, direction):
    """Operator names of an architecture's forward (0) or backward (1) graph, in id order."""
    out = []
    while True:
        r = lib.dh_op_name(arch, direction, len(out))
        if r is None:
            return out
        out.append(r.decode())


class DhelixError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libdhelix error %d: %s" % (code, msg))
        self.code = code


class dh_layer_config(C.Structure):
    _fields_ = [("arch", C.c_int), ("dtype", C.c_int), ("batch", C.c_int), ("seq", C.c_int), ("hidden", C.c_int),
                ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int), ("ffn", C.c_int),
                ("eps", C.c_float), ("rope_base", C.c_float), ("n_ranks", C.c_int), ("comm_blocks", C.c_int),
                ("n_experts", C.c_int), ("n_local_experts", C.c_int), ("cp_ranks", C.c_int), ("cp_rank", C.c_int),
                ("cross_blocks", C.c_int), ("rope_pairing", C.c_int), ("gelu_form", C.c_int)]


class dh_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g1", "Wqkv", "Wo", "g2", "Wgu", "Wd", "b1", "bqkv", "bo", "b2", "bfc1", "bfc2")]


class dh_wgrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dg1", "dWqkv", "dWo", "dg2", "dWgu", "dWd", "db1", "dbqkv", "dbo", "db2", "dbfc1",
                                          "dbfc2")]


class dh_fwd_args(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("x", "out", "saved", "peers_ar1", "peers_ar2", "peers_ag1", "peers_ag2", "logits",
                                          "peers_kv")]


class dh_bwd_args(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dout", "dx", "x", "saved", "peers_ar3", "peers_ar4", "peers_ag3", "peers_ag4",
                                          "dlogits", "peers_dkv", "dkv_peers")]


class dh_op_graph(C.Structure):
    _fields_ = [("n_ops", C.c_int), ("is_comm", C.c_int * DH_MAX_OPS), ("n_deps", C.c_int),
                ("dep_src", C.c_int * DH_MAX_DEPS), ("dep_dst", C.c_int * DH_MAX_DEPS), ("side_ok", C.c_int * DH_MAX_OPS),
                ("like_other", C.c_int * DH_MAX_OPS)]


class dh_lanes(C.Structure):
    _fields_ = [("comm_alpha", C.c_int), ("comm_beta", C.c_int), ("cross", C.c_int)]


class dh_search_info(C.Structure):
    _fields_ = [("orders_fwd_total", C.c_longlong), ("orders_bwd_total", C.c_longlong), ("orders_fwd_tried", C.c_int),
                ("orders_bwd_tried", C.c_int), ("truncated", C.c_int), ("refined", C.c_int)]


class dh_overlap_table(C.Structure):
    _fields_ = [("n_fwd", C.c_int), ("n_bwd", C.c_int), ("t_fwd", C.c_double * DH_MAX_OPS),
                ("t_bwd", C.c_double * DH_MAX_OPS), ("rate_fwd", (C.c_double * DH_MAX_OPS) * DH_MAX_OPS),
                ("rate_bwd", (C.c_double * DH_MAX_OPS) * DH_MAX_OPS), ("p_pair", (C.c_double * DH_MAX_OPS) * DH_MAX_OPS),
                ("oef", (C.c_double * DH_MAX_OPS) * DH_MAX_OPS)]


class dh_seg_pair(C.Structure):
    _fields_ = [("f_begin", C.c_int), ("f_end", C.c_int), ("b_begin", C.c_int), ("b_end", C.c_int)]


MOE_TABLES = ("rank", "dest", "src_tok", "send_of_recv", "recv_of_send", "counts", "offsets", "recv_start", "group_rows")


class dh_moe_tables(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in MOE_TABLES]


class dh_cp_move(C.Structure):
    _fields_ = [("src", C.c_void_p), ("dst", C.c_void_p), ("src_ld", C.c_int), ("src_seq_rows", C.c_int), ("src_row0", C.c_int),
                ("dst_ld", C.c_int), ("dst_seq_rows", C.c_int), ("dst_row0", C.c_int)]


class dh_stack_fwd(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("x", "out", "peers_ar1", "peers_ar2")]


class dh_stack_bwd(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dout", "dx", "peers_ar3", "peers_ar4")]


class dh_plan(C.Structure):
    _fields_ = [("n_fwd", C.c_int), ("n_bwd", C.c_int), ("n_pairs", C.c_int), ("fwd_order", C.c_int * DH_MAX_OPS),
                ("bwd_order", C.c_int * DH_MAX_OPS), ("pairs", dh_seg_pair * (2 * DH_MAX_OPS)),
                ("bwd_side", C.c_int * DH_MAX_OPS)]


# Every symbol include/dhelix.h declares, with its C signature.
_P, _I, _Z, _D, _F = C.c_void_p, C.c_int, C.c_size_t, C.c_double, C.c_float
SIGNATURES = {
    "dh_last_error": (C.c_char_p, []),
    "dh_layer_create": (_I, [C.POINTER(dh_layer_config), C.POINTER(_P)]),
    "dh_layer_destroy": (None, [_P]),
    "dh_layer_bind_weights": (_I, [_P, C.POINTER(dh_weights)]),
    "dh_layer_bind_wgrads": (_I, [_P, C.POINTER(dh_wgrads)]),
    "dh_layer_saved_bytes": (_Z, [_P]),
    "dh_layer_workspace_bytes": (_Z, [_P, _I]),
    "dh_layer_fwd": (_I, [_P, C.POINTER(dh_fwd_args), _P, _Z, _P]),
    "dh_layer_bwd": (_I, [_P, C.POINTER(dh_bwd_args), _P, _Z, _P]),
    "dh_layer_op_graph": (_I, [_P, _I, C.POINTER(dh_op_graph)]),
    "dh_op_name": (C.c_char_p, [_I, _I, _I]),
    "dh_oef": (_D, [_D, _D, _D]),
    "dh_segment_cost": (_D, [C.POINTER(dh_overlap_table), C.POINTER(_I), _I, C.POINTER(_I), _I]),
    "dh_profile_pairs": (_I, [_P, C.POINTER(dh_fwd_args), C.POINTER(dh_bwd_args), _P, _Z, _P, _P, _P, _I,
                              C.POINTER(dh_overlap_table)]),
    "dh_pair_dp": (_I, [C.POINTER(_D), _I, C.POINTER(_D), _I, C.POINTER(_D), C.POINTER(_D), C.POINTER(_I), C.POINTER(_I)]),
    "dh_plan_search": (_I, [C.POINTER(dh_op_graph), C.POINTER(dh_op_graph), C.POINTER(dh_overlap_table), _D, _I,
                            C.POINTER(dh_plan), C.POINTER(_D)]),
    "dh_plan_validate": (_I, [C.POINTER(dh_op_graph), C.POINTER(dh_op_graph), C.POINTER(dh_plan)]),
    "dh_plan_count_orders": (C.c_longlong, [C.POINTER(dh_op_graph), C.c_longlong]),
    "dh_plan_cost": (_D, [C.POINTER(dh_op_graph), C.POINTER(dh_op_graph), C.POINTER(dh_overlap_table), C.POINTER(dh_plan),
                          C.POINTER(dh_lanes), _D]),
    "dh_plan_search_lanes": (_I, [C.POINTER(dh_op_graph), C.POINTER(dh_op_graph), C.POINTER(dh_overlap_table),
                                  C.POINTER(dh_lanes), _D, _I, C.POINTER(dh_plan), C.POINTER(_D), C.POINTER(dh_search_info)]),
    "dh_profile_solo": (_I, [_P, C.POINTER(dh_fwd_args), C.POINTER(dh_bwd_args), _P, _Z, _P, _P, _P, _I, C.POINTER(_D), C.POINTER(_D)]),
    "dh_layer_set_beta_comm_stream": (_I, [_P, _P]),
    "dh_layer_set_comm_blocks": (_I, [_P, _I]),
    "dh_plan_round_robin": (_I, [C.POINTER(dh_op_graph), C.POINTER(dh_op_graph), C.POINTER(dh_plan)]),
    "dh_plan_sequential": (_I, [_P, C.POINTER(dh_plan)]),
    "dh_si_step": (_I, [_P, C.POINTER(dh_fwd_args), C.POINTER(dh_bwd_args), C.POINTER(dh_plan), _P, _Z, _P, _P, _P]),
    "dh_si_step_layers": (_I, [_P, _P, C.POINTER(dh_fwd_args), C.POINTER(dh_bwd_args), C.POINTER(dh_plan), _P, _Z, _P, _P, _P]),
    "dh_stack_create": (_I, [C.POINTER(dh_layer_config), _I, C.POINTER(_P)]),
    "dh_stack_destroy": (None, [_P]),
    "dh_stack_layer": (_P, [_P, _I]),
    "dh_stack_arena_bytes": (_Z, [_P]),
    "dh_stack_unshared_bytes": (_Z, [_P]),
    "dh_stack_workspace_bytes": (_Z, [_P]),
    "dh_stack_phase": (_I, [_P, C.POINTER(dh_stack_fwd), C.POINTER(dh_stack_bwd), C.POINTER(dh_plan), _P, _Z, _P, _Z, _P, _P, _P]),
    "dh_si_graph_create": (_I, [_P, C.POINTER(dh_fwd_args), C.POINTER(dh_bwd_args), C.POINTER(dh_plan), _P, _Z, _P, _P,
                                C.POINTER(_P)]),
    "dh_si_graph_launch": (_I, [_P, _P]),
    "dh_si_graph_destroy": (None, [_P]),
    "dh_comm_standin": (_I, [_I, _I, C.POINTER(_P), _P, _Z, _I, _I, _P]),
    "dh_cp_exchange": (_I, [_I, _I, C.POINTER(dh_cp_move), _I, _I, _I, _I, _P]),
    "dh_cp_grad_reduce": (_I, [_I, C.POINTER(dh_cp_move), _I, C.POINTER(_P), _I, _I, _I, _I, _P]),
    "dh_layer_set_cross_stream": (_I, [_P, _P]),
    "dh_stream_create_masked": (_I, [_I, C.POINTER(_P)]),
    "dh_stream_destroy": (_I, [_P]),
    "dh_gemm": (_I, [_I, _I, _I, _I, _I, _I, _P, _P, _P, _I, _P, _Z, _P]),
    "dh_gemm_workspace_bytes": (_Z, [_I, _I, _I, _I, _I, _I]),
    "dh_rmsnorm_fwd": (_I, [_I, _I, _I, _P, _P, _P, _F, _P, _P, _P, _P]),
    "dh_rmsnorm_bwd": (_I, [_I, _I, _I, _P, _P, _P, _P, _P, _P, _P, _P, _Z, _P]),
    "dh_rmsnorm_bwd_ws_bytes": (_Z, [_I, _I]),
    "dh_rmsnorm_bwd_noalloc": (_I, [_I, _I, _I, _P, _P, _P, _P, _P, _P, _P, _P]),
    "dh_rmsnorm_bwd_noalloc_max_bytes": (_Z, []),
    "dh_rope": (_I, [_I, _I, _I, _I, _I, _I, _F, _I, _P, _P]),
    "dh_rope_at": (_I, [_I, _I, _I, _I, _I, _I, _I, _F, _I, _P, _P]),
    "dh_rope_pairs": (_I, [_I, _I, _I, _I, _I, _I, _I, _I, _F, _I, _P, _P]),
    "dh_swiglu_fwd": (_I, [_I, _I, _I, _P, _P, _P]),
    "dh_swiglu_bwd": (_I, [_I, _I, _I, _P, _P, _P, _P]),
    "dh_layer_set_fused_activation": (_I, [_P, _I]),
    "dh_layer_set_fused_collective": (_I, [_P, _I]),
    "dh_gemm_allreduce_fits": (_I, [_I, _I, _I, _I, _I]),
    "dh_gemm_allreduce": (_I, [_I, _I, _I, _I, _I, _P, _P, _P, _I, _I, C.POINTER(_P), _P, _Z, _I, _P]),
    "dh_gemm_swiglu_fwd_fits": (_I, [_I, _I, _I]),
    "dh_gemm_swiglu_fwd": (_I, [_I, _I, _I, _P, _P, _P, _P, _P]),
    "dh_gemm_swiglu_bwd_fits": (_I, [_I, _I, _I]),
    "dh_gemm_swiglu_bwd": (_I, [_I, _I, _I, _P, _P, _P, _P, _P]),
    "dh_add": (_I, [_I, _Z, _P, _P, _P, _P]),
    "dh_attn_fwd": (_I, [_I, _I, _I, _I, _I, _I, _P, _P, _P, _P, _Z, _P]),
    "dh_attn_fwd_workspace_bytes": (_Z, [_I, _I, _I, _I, _I, _I]),
    "dh_attn_bwd": (_I, [_I, _I, _I, _I, _I, _I, _P, _P, _P, _P, _P, _P, _P, _Z, _P]),
    "dh_attn_bwd_workspace_bytes": (_Z, [_I, _I, _I, _I, _I, _I]),
    "dh_attn_ctx_fwd": (_I, [_I, _I, _I, _I, _I, _I, _I, _P, _P, _P, _P, _P, _Z, _P]),
    "dh_attn_ctx_fwd_workspace_bytes": (_Z, [_I, _I, _I, _I, _I, _I, _I]),
    "dh_attn_ctx_bwd": (_I, [_I, _I, _I, _I, _I, _I, _I, _P, _P, _P, _P, _P, _P, _P, _P, _P, _Z, _P]),
    "dh_attn_ctx_bwd_workspace_bytes": (_Z, [_I, _I, _I, _I, _I, _I, _I]),
    "dh_moe_route": (_I, [_I, _I, _P, _P, _P, _P]),
    "dh_moe_route_bwd": (_I, [_I, _I, _P, _P, _P, _P, _P]),
    "dh_moe_plan": (_I, [_I, _I, _I, _P, C.POINTER(dh_moe_tables), _P]),
    "dh_moe_gather_rows": (_I, [_I, _I, _I, _P, _P, _P, _I, _P]),
    "dh_moe_combine": (_I, [_I, _I, _I, _P, _P, _P, _P, _P, _P]),
    "dh_moe_combine_bwd": (_I, [_I, _I, _I, _P, _P, _P, _P, _P, _P, _P]),
    "dh_gemm_grouped": (_I, [_I, _I, _I, _P, _I, _I, _I, _P, _P, _P, _P]),
    "dh_gemm_bias": (_I, [_I, _I, _I, _I, _I, _I, _P, _P, _P, _P, _I, _P, _Z, _P]),
    "dh_layernorm_fwd": (_I, [_I, _I, _I, _P, _P, _P, _P, _P, _F, _P, _P, _P, _P, _P]),
    "dh_layernorm_bwd": (_I, [_I, _I, _I, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _Z, _P]),
    "dh_layernorm_bwd_ws_bytes": (_Z, [_I, _I]),
    "dh_gelu_fwd": (_I, [_I, _Z, _P, _P, _P]),
    "dh_gelu_bwd": (_I, [_I, _Z, _P, _P, _P, _P]),
    "dh_gelu_fwd_form": (_I, [_I, _I, _Z, _P, _P, _P]),
    "dh_gelu_bwd_form": (_I, [_I, _I, _Z, _P, _P, _P, _P]),
    "dh_bias_residual_add": (_I, [_I, _I, _I, _P, _P, _P, _P, _P]),
    "dh_colsum": (_I, [_I, _I, _I, _P, _P, _P, _Z, _P]),
    "dh_colsum_ws_bytes": (_Z, [_I, _I]),
}
for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def _check(rc):
    if rc != DH_OK:
        raise DhelixError(rc, lib.dh_last_error().decode())


def dh_last_error():
    return lib.dh_last_error().decode()


def dh_layer_create(**cfg):
    c = dh_layer_config(**cfg)
    h = _P()
    _check(lib.dh_layer_create(C.byref(c), C.byref(h)))
    return h


def dh_layer_destroy(layer):
    lib.dh_layer_destroy(layer)


def dh_layer_bind_weights(layer, **w):
    s = dh_weights(**{k: _ptr(v) for k, v in w.items()})
    _check(lib.dh_layer_bind_weights(layer, C.byref(s)))


def dh_layer_bind_wgrads(layer, **g):
    s = dh_wgrads(**{k: _ptr(v) for k, v in g.items()})
    _check(lib.dh_layer_bind_wgrads(layer, C.byref(s)))


def dh_layer_saved_bytes(layer):
    return lib.dh_layer_saved_bytes(layer)


def dh_layer_workspace_bytes(layer, kind):
    return lib.dh_layer_workspace_bytes(layer, kind)


def fwd_args(x, out, saved, peers_ar1=None, peers_ar2=None, peers_ag1=None, peers_ag2=None, logits=None, peers_kv=None):
    return dh_fwd_args(_ptr(x), _ptr(out), _ptr(saved), _ptr(peers_ar1), _ptr(peers_ar2), _ptr(peers_ag1), _ptr(peers_ag2),
                       _ptr(logits), _ptr(peers_kv))


def bwd_args(dout, dx, x, saved, peers_ar3=None, peers_ar4=None, peers_ag3=None, peers_ag4=None, dlogits=None, peers_dkv=None,
             dkv_peers=None):
    return dh_bwd_args(_ptr(dout), _ptr(dx), _ptr(x), _ptr(saved), _ptr(peers_ar3), _ptr(peers_ar4), _ptr(peers_ag3),
                       _ptr(peers_ag4), _ptr(dlogits), _ptr(peers_dkv), _ptr(dkv_peers))


def dh_layer_fwd(layer, args, ws, ws_bytes, stream=None):
    _check(lib.dh_layer_fwd(layer, C.byref(args), _ptr(ws), ws_bytes, _stream(stream)))


def dh_layer_bwd(layer, args, ws, ws_bytes, stream=None):
    _check(lib.dh_layer_bwd(layer, C.byref(args), _ptr(ws), ws_bytes, _stream(stream)))


def dh_layer_op_graph(layer, direction):
    g = dh_op_graph()
    _check(lib.dh_layer_op_graph(layer, direction, C.byref(g)))
    return g


def dh_op_name(arch, direction, op):
    r = lib.dh_op_name(arch, direction, op)
    return r.decode() if r else None


def dh_oef(t_i, t_j, p_ij):
    return lib.dh_oef(t_i, t_j, p_ij)


def make_table(t_fwd, t_bwd, rate_fwd, rate_bwd):
    t = dh_overlap_table()
    t.n_fwd, t.n_bwd = len(t_fwd), len(t_bwd)
    for i, v in enumerate(t_fwd):
        t.t_fwd[i] = v
    for j, v in enumerate(t_bwd):
        t.t_bwd[j] = v
    for i in range(len(t_fwd)):
        for j in range(len(t_bwd)):
            t.rate_fwd[i][j] = rate_fwd[i][j]
            t.rate_bwd[i][j] = rate_bwd[i][j]
    return t


def make_graph(n_ops, deps, comm=(), side_ok=(), like=None):
    """like: {op: id of the like operator of the other direction's graph}."""
    g = dh_op_graph()
    g.n_ops = n_ops
    g.n_deps = len(deps)
    for e, (s, d) in enumerate(deps):
        g.dep_src[e], g.dep_dst[e] = s, d
    for c in comm:
        g.is_comm[c] = 1
    for c in side_ok:
        g.side_ok[c] = 1
    for op, other in (like or {}).items():
        g.like_other[op] = other + 1
    return g


def with_side(plan, side_ops):
    """A copy of the plan whose backward operators `side_ops` run beside their strand."""
    q = dh_plan.from_buffer_copy(plan)
    for op in range(DH_MAX_OPS):
        q.bwd_side[op] = 1 if op in side_ops else 0
    return q


def make_plan(fwd_order, bwd_order, pairs, side=()):
    p = dh_plan()
    for op in side:
        p.bwd_side[op] = 1
    p.n_fwd, p.n_bwd, p.n_pairs = len(fwd_order), len(bwd_order), len(pairs)
    for i, v in enumerate(fwd_order):
        p.fwd_order[i] = v
    for j, v in enumerate(bwd_order):
        p.bwd_order[j] = v
    for k, (a, b, c, d) in enumerate(pairs):
        p.pairs[k] = dh_seg_pair(a, b, c, d)
    return p


def plan_to_py(p):
    return (list(p.fwd_order[: p.n_fwd]), list(p.bwd_order[: p.n_bwd]),
            [(q.f_begin, q.f_end, q.b_begin, q.b_end) for q in p.pairs[: p.n_pairs]])


def dh_segment_cost(table, seg_f, seg_b):
    a = (C.c_int * max(1, len(seg_f)))(*seg_f)
    b = (C.c_int * max(1, len(seg_b)))(*seg_b)
    r = lib.dh_segment_cost(C.byref(table), a, len(seg_f), b, len(seg_b))
    if r < 0:
        raise DhelixError(int(r), dh_last_error())
    return r


def dh_pair_dp(p_f, p_b, p_fb):
    nf, nb = len(p_f), len(p_b)
    a = (C.c_double * max(1, nf))(*p_f)
    b = (C.c_double * max(1, nb))(*p_b)
    flat = [p_fb[i][j] for i in range(nf) for j in range(nb)]
    c = (C.c_double * max(1, nf * nb))(*flat)
    t = C.c_double()
    steps = (C.c_int * (2 * (nf + nb) + 2))()
    n = C.c_int()
    _check(lib.dh_pair_dp(a, nf, b, nb, c, C.byref(t), steps, C.byref(n)))
    return t.value, [(steps[2 * k] if steps[2 * k] >= 0 else None, steps[2 * k + 1] if steps[2 * k + 1] >= 0 else None)
                     for k in range(n.value)]


def dh_plan_search(fwd_graph, bwd_graph, table, barrier_cost=0.0, max_orders=0):
    p = dh_plan()
    m = C.c_double()
    _check(lib.dh_plan_search(C.byref(fwd_graph), C.byref(bwd_graph), C.byref(table), barrier_cost, max_orders,
                              C.byref(p), C.byref(m)))
    return p, m.value


def dh_plan_count_orders(graph, cap=1 << 40):
    r = lib.dh_plan_count_orders(C.byref(graph), cap)
    if r < 0:
        raise DhelixError(int(r), dh_last_error())
    return r


def lanes(comm_alpha=0, comm_beta=0, cross=0):
    return dh_lanes(comm_alpha, comm_beta, cross)


def dh_plan_cost(fwd_graph, bwd_graph, table, plan, lane_cfg, barrier_cost=0.0):
    r = lib.dh_plan_cost(C.byref(fwd_graph), C.byref(bwd_graph), C.byref(table), C.byref(plan), C.byref(lane_cfg), barrier_cost)
    if r < 0:
        raise DhelixError(int(r), dh_last_error())
    return r


def dh_plan_search_lanes(fwd_graph, bwd_graph, table, lane_cfg, barrier_cost=0.0, max_orders=0):
    """Returns (plan, predicted makespan, dh_search_info)."""
    p, m, info = dh_plan(), C.c_double(), dh_search_info()
    _check(lib.dh_plan_search_lanes(C.byref(fwd_graph), C.byref(bwd_graph), C.byref(table), C.byref(lane_cfg), barrier_cost,
                                    max_orders, C.byref(p), C.byref(m), C.byref(info)))
    return p, m.value, info


def dh_profile_solo(layer, alpha, beta, ws, ws_bytes, stream_alpha, stream_beta, comm_stream, reps=20):
    """Returns (t_fwd, t_bwd): lists of DH_MAX_OPS solo times in seconds."""
    tf, tb = (C.c_double * DH_MAX_OPS)(), (C.c_double * DH_MAX_OPS)()
    _check(lib.dh_profile_solo(layer, C.byref(alpha), C.byref(beta), _ptr(ws), ws_bytes, _stream(stream_alpha),
                               _stream(stream_beta), _stream(comm_stream), reps, tf, tb))
    return list(tf), list(tb)


def dh_layer_set_beta_comm_stream(layer, stream):
    _check(lib.dh_layer_set_beta_comm_stream(layer, _stream(stream)))


def dh_layer_set_comm_blocks(layer, comm_blocks):
    _check(lib.dh_layer_set_comm_blocks(layer, comm_blocks))


def dh_plan_validate(fwd_graph, bwd_graph, plan):
    _check(lib.dh_plan_validate(C.byref(fwd_graph), C.byref(bwd_graph), C.byref(plan)))


def dh_plan_round_robin(fwd_graph, bwd_graph):
    p = dh_plan()
    _check(lib.dh_plan_round_robin(C.byref(fwd_graph), C.byref(bwd_graph), C.byref(p)))
    return p


def dh_plan_sequential(layer):
    p = dh_plan()
    _check(lib.dh_plan_sequential(layer, C.byref(p)))
    return p


def dh_profile_pairs(layer, alpha, beta, ws, ws_bytes, stream_alpha, stream_beta, comm_stream, reps=5):
    t = dh_overlap_table()
    _check(lib.dh_profile_pairs(layer, C.byref(alpha), C.byref(beta), _ptr(ws), ws_bytes, _stream(stream_alpha),
                                _stream(stream_beta), _stream(comm_stream), reps, C.byref(t)))
    return t


def dh_si_step(layer, alpha, beta, plan, ws, ws_bytes, stream_alpha, stream_beta, stream_comm=None):
    _check(lib.dh_si_step(layer, C.byref(alpha), C.byref(beta), C.byref(plan), _ptr(ws), ws_bytes,
                          _stream(stream_alpha), _stream(stream_beta), _stream(stream_comm)))


def dh_si_step_layers(layer_alpha, layer_beta, alpha, beta, plan, ws, ws_bytes, stream_alpha, stream_beta, stream_comm=None):
    _check(lib.dh_si_step_layers(layer_alpha, layer_beta, C.byref(alpha), C.byref(beta), C.byref(plan), _ptr(ws), ws_bytes,
                                 _stream(stream_alpha), _stream(stream_beta), _stream(stream_comm)))


def dh_stack_create(n_layers, **cfg):
    c = dh_layer_config(**cfg)
    h = _P()
    _check(lib.dh_stack_create(C.byref(c), n_layers, C.byref(h)))
    return h


def dh_stack_destroy(stack):
    lib.dh_stack_destroy(stack)


def dh_stack_layer(stack, i):
    return _P(lib.dh_stack_layer(stack, i))


def dh_stack_arena_bytes(stack):
    return lib.dh_stack_arena_bytes(stack)


def dh_stack_unshared_bytes(stack):
    return lib.dh_stack_unshared_bytes(stack)


def dh_stack_workspace_bytes(stack):
    return lib.dh_stack_workspace_bytes(stack)


def dh_stack_phase(stack, alpha, beta, plan, arena, arena_bytes, ws, ws_bytes, stream_alpha=None, stream_beta=None,
                   stream_comm=None):
    """alpha: (x, out, peers_ar1, peers_ar2) or None; beta: (dout, dx, peers_ar3, peers_ar4) or None."""
    a = dh_stack_fwd(*[_ptr(t) for t in alpha]) if alpha is not None else None
    b = dh_stack_bwd(*[_ptr(t) for t in beta]) if beta is not None else None
    _check(lib.dh_stack_phase(stack, C.byref(a) if a is not None else None, C.byref(b) if b is not None else None,
                              C.byref(plan) if plan is not None else None, _ptr(arena), arena_bytes, _ptr(ws), ws_bytes,
                              _stream(stream_alpha), _stream(stream_beta), _stream(stream_comm)))


def dh_si_graph_create(layer, alpha, beta, plan, ws, ws_bytes, stream_alpha, stream_beta):
    g = _P()
    _check(lib.dh_si_graph_create(layer, C.byref(alpha), C.byref(beta), C.byref(plan), _ptr(ws), ws_bytes,
                                  _stream(stream_alpha), _stream(stream_beta), C.byref(g)))
    return g


def dh_si_graph_launch(graph, stream=None):
    _check(lib.dh_si_graph_launch(graph, _stream(stream)))


def dh_si_graph_destroy(graph):
    lib.dh_si_graph_destroy(graph)


def dh_comm_standin(kind, parts, out, elems, dtype, n_blocks=0, stream=None):
    arr = (_P * len(parts))(*[_ptr(p) for p in parts])
    _check(lib.dh_comm_standin(kind, len(parts), arr, _ptr(out), elems, dtype, n_blocks, _stream(stream)))


def cp_move(src, dst, src_ld, src_seq_rows, src_row0, dst_ld, dst_seq_rows, dst_row0):
    return dh_cp_move(_ptr(src), _ptr(dst), src_ld, src_seq_rows, src_row0, dst_ld, dst_seq_rows, dst_row0)


def dh_cp_exchange(dtype, moves, batch, rows, width, n_blocks=0, stream=None):
    arr = (dh_cp_move * max(len(moves), 1))(*moves)
    _check(lib.dh_cp_exchange(dtype, len(moves), arr, batch, rows, width, n_blocks, _stream(stream)))


def dh_cp_grad_reduce(dtype, own, peers, batch, rows, width, n_blocks=0, stream=None):
    arr = (_P * max(len(peers), 1))(*[_ptr(p) for p in peers])
    _check(lib.dh_cp_grad_reduce(dtype, C.byref(own), len(peers), arr, batch, rows, width, n_blocks, _stream(stream)))


def dh_layer_set_cross_stream(layer, stream):
    _check(lib.dh_layer_set_cross_stream(layer, _stream(stream)))


def dh_stream_create_masked(n_cus):
    s = _P()
    _check(lib.dh_stream_create_masked(n_cus, C.byref(s)))
    return s.value


def dh_stream_destroy(stream):
    _check(lib.dh_stream_destroy(stream))


def dh_gemm(dtype, trans_a, trans_b, M, N, K, A, B, Cout, out_f32_accumulate=False, ws=None, ws_bytes=0, stream=None):
    _check(lib.dh_gemm(dtype, int(trans_a), int(trans_b), M, N, K, _ptr(A), _ptr(B), _ptr(Cout), int(out_f32_accumulate),
                       _ptr(ws), ws_bytes, _stream(stream)))


def dh_gemm_workspace_bytes(dtype, trans_a, trans_b, M, N, K):
    return lib.dh_gemm_workspace_bytes(dtype, int(trans_a), int(trans_b), M, N, K)


def dh_rmsnorm_fwd(dtype, T, H, x, residual, gamma, eps, x_out, h, rstd, stream=None):
    _check(lib.dh_rmsnorm_fwd(dtype, T, H, _ptr(x), _ptr(residual), _ptr(gamma), eps, _ptr(x_out), _ptr(h), _ptr(rstd),
                              _stream(stream)))


def dh_rmsnorm_bwd_ws_bytes(T, H):
    return lib.dh_rmsnorm_bwd_ws_bytes(T, H)


def dh_rmsnorm_bwd(dtype, T, H, dy, x, gamma, rstd, dres, dx, dgamma, ws, ws_bytes, stream=None):
    _check(lib.dh_rmsnorm_bwd(dtype, T, H, _ptr(dy), _ptr(x), _ptr(gamma), _ptr(rstd), _ptr(dres), _ptr(dx),
                              _ptr(dgamma), _ptr(ws), ws_bytes, _stream(stream)))


def dh_rmsnorm_bwd_noalloc(dtype, T, H, dy, x, gamma, rstd, dres, dx, dgamma, stream=None):
    _check(lib.dh_rmsnorm_bwd_noalloc(dtype, T, H, _ptr(dy), _ptr(x), _ptr(gamma), _ptr(rstd), _ptr(dres), _ptr(dx),
                                      _ptr(dgamma), _stream(stream)))


def dh_rmsnorm_bwd_noalloc_max_bytes():
    return lib.dh_rmsnorm_bwd_noalloc_max_bytes()


def dh_rope(dtype, T, seq, n_heads, head_dim, row_stride, base, inverse, t, stream=None):
    _check(lib.dh_rope(dtype, T, seq, n_heads, head_dim, row_stride, base, int(inverse), _ptr(t), _stream(stream)))


def dh_swiglu_fwd(dtype, T, F, gu, a, stream=None):
    _check(lib.dh_swiglu_fwd(dtype, T, F, _ptr(gu), _ptr(a), _stream(stream)))


def dh_swiglu_bwd(dtype, T, F, gu, da, dgu, stream=None):
    _check(lib.dh_swiglu_bwd(dtype, T, F, _ptr(gu), _ptr(da), _ptr(dgu), _stream(stream)))


def dh_layer_set_fused_activation(layer, enable):
    """Returns the bit mask of what is fused afterwards (1 forward, 2 backward)."""
    rc = lib.dh_layer_set_fused_activation(layer, 3 if enable is True else int(enable))
    if rc < 0:
        _check(rc)
    return rc


def dh_layer_set_fused_collective(layer, mask):
    """Returns the mask in force afterwards (1: B_AR3 carries B_FC1_WGRAD, 2: B_AR4 carries B_QKV_WGRAD)."""
    rc = lib.dh_layer_set_fused_collective(layer, int(mask))
    if rc < 0:
        _check(rc)
    return rc


def dh_gemm_allreduce_fits(trans_a, trans_b, M, N, K):
    return bool(lib.dh_gemm_allreduce_fits(trans_a, trans_b, M, N, K))


def dh_gemm_allreduce(trans_a, trans_b, M, N, K, A, B, Cmat, out_f32_accumulate, parts, ar_out, ar_elems, n_blocks, stream=None):
    arr = (_P * len(parts))(*[_ptr(q) for q in parts])
    _check(lib.dh_gemm_allreduce(trans_a, trans_b, M, N, K, _ptr(A), _ptr(B), _ptr(Cmat), 1 if out_f32_accumulate else 0,
                                 len(parts), arr, _ptr(ar_out), ar_elems, n_blocks, _stream(stream)))


def dh_gemm_swiglu_fwd_fits(T, F, H):
    return bool(lib.dh_gemm_swiglu_fwd_fits(T, F, H))


def dh_gemm_swiglu_fwd(T, F, H, x, w_gate_up, gu, a, stream=None):
    _check(lib.dh_gemm_swiglu_fwd(T, F, H, _ptr(x), _ptr(w_gate_up), _ptr(gu), _ptr(a), _stream(stream)))


def dh_gemm_swiglu_bwd_fits(T, F, H):
    return bool(lib.dh_gemm_swiglu_bwd_fits(T, F, H))


def dh_gemm_swiglu_bwd(T, F, H, dy, w_down, gu, dgu, stream=None):
    _check(lib.dh_gemm_swiglu_bwd(T, F, H, _ptr(dy), _ptr(w_down), _ptr(gu), _ptr(dgu), _stream(stream)))


def dh_add(dtype, n, a, b, out, stream=None):
    _check(lib.dh_add(dtype, n, _ptr(a), _ptr(b), _ptr(out), _stream(stream)))


def dh_rope_at(dtype, T, seq, pos0, n_heads, head_dim, row_stride, base, inverse, t, stream=None):
    _check(lib.dh_rope_at(dtype, T, seq, pos0, n_heads, head_dim, row_stride, base, int(inverse), _ptr(t), _stream(stream)))


def dh_attn_ctx_fwd(dtype, batch, seq, q_off, nq, nkv, d, qkv, kv, o, lse, ws=None, ws_bytes=0, stream=None):
    _check(lib.dh_attn_ctx_fwd(dtype, batch, seq, q_off, nq, nkv, d, _ptr(qkv), _ptr(kv), _ptr(o), _ptr(lse), _ptr(ws), ws_bytes,
                               _stream(stream)))


def dh_attn_ctx_fwd_workspace_bytes(dtype, batch, seq, q_off, nq, nkv, d):
    return lib.dh_attn_ctx_fwd_workspace_bytes(dtype, batch, seq, q_off, nq, nkv, d)


def dh_attn_ctx_bwd(dtype, batch, seq, q_off, nq, nkv, d, qkv, kv, o, dout, lse, dqkv, dkv, delta, ws=None, ws_bytes=0, stream=None):
    _check(lib.dh_attn_ctx_bwd(dtype, batch, seq, q_off, nq, nkv, d, _ptr(qkv), _ptr(kv), _ptr(o), _ptr(dout), _ptr(lse), _ptr(dqkv),
                               _ptr(dkv), _ptr(delta), _ptr(ws), ws_bytes, _stream(stream)))


def dh_attn_ctx_bwd_workspace_bytes(dtype, batch, seq, q_off, nq, nkv, d):
    return lib.dh_attn_ctx_bwd_workspace_bytes(dtype, batch, seq, q_off, nq, nkv, d)


def dh_attn_fwd(dtype, batch, seq, nq, nkv, d, qkv, o, lse, ws=None, ws_bytes=0, stream=None):
    _check(lib.dh_attn_fwd(dtype, batch, seq, nq, nkv, d, _ptr(qkv), _ptr(o), _ptr(lse), _ptr(ws), ws_bytes, _stream(stream)))


def dh_attn_fwd_workspace_bytes(dtype, batch, seq, nq, nkv, d):
    return lib.dh_attn_fwd_workspace_bytes(dtype, batch, seq, nq, nkv, d)


def dh_attn_bwd(dtype, batch, seq, nq, nkv, d, qkv, o, dout, lse, dqkv, delta, ws=None, ws_bytes=0, stream=None):
    _check(lib.dh_attn_bwd(dtype, batch, seq, nq, nkv, d, _ptr(qkv), _ptr(o), _ptr(dout), _ptr(lse), _ptr(dqkv),
                           _ptr(delta), _ptr(ws), ws_bytes, _stream(stream)))


def dh_attn_bwd_workspace_bytes(dtype, batch, seq, nq, nkv, d):
    return lib.dh_attn_bwd_workspace_bytes(dtype, batch, seq, nq, nkv, d)


def dh_moe_route(T, E, logits, idx, prob, stream=None):
    _check(lib.dh_moe_route(T, E, _ptr(logits), _ptr(idx), _ptr(prob), _stream(stream)))


def dh_moe_route_bwd(T, E, dprob, idx, prob, dlogits, stream=None):
    _check(lib.dh_moe_route_bwd(T, E, _ptr(dprob), _ptr(idx), _ptr(prob), _ptr(dlogits), _stream(stream)))


def moe_tables(**tensors):
    """dh_moe_tables from int32 device tensors named as the struct's fields."""
    return dh_moe_tables(**{n: _ptr(tensors[n]) for n in MOE_TABLES})


def dh_moe_plan(T, E, n_local, idx, tables, stream=None):
    _check(lib.dh_moe_plan(T, E, n_local, _ptr(idx), C.byref(tables), _stream(stream)))


def dh_moe_gather_rows(dtype, n_rows, H, inp, row_map, out, n_blocks=0, stream=None):
    _check(lib.dh_moe_gather_rows(dtype, n_rows, H, _ptr(inp), _ptr(row_map), _ptr(out), n_blocks, _stream(stream)))


def dh_moe_combine(dtype, T, H, yp, dest, prob, residual, y, stream=None):
    _check(lib.dh_moe_combine(dtype, T, H, _ptr(yp), _ptr(dest), _ptr(prob), _ptr(residual), _ptr(y), _stream(stream)))


def dh_moe_combine_bwd(dtype, T, H, dy, yp, dest, prob, dyp, dprob, stream=None):
    _check(lib.dh_moe_combine_bwd(dtype, T, H, _ptr(dy), _ptr(yp), _ptr(dest), _ptr(prob), _ptr(dyp), _ptr(dprob),
                                  _stream(stream)))


def dh_gemm_grouped(dtype, mode, n_groups, group_rows, max_rows, dim_a, dim_b, A, B, Cout, stream=None):
    _check(lib.dh_gemm_grouped(dtype, mode, n_groups, _ptr(group_rows), max_rows, dim_a, dim_b, _ptr(A), _ptr(B), _ptr(Cout),
                               _stream(stream)))


def dh_gemm_bias(dtype, trans_a, trans_b, M, N, K, A, B, bias, Cout, out_f32_accumulate=False, ws=None, ws_bytes=0, stream=None):
    _check(lib.dh_gemm_bias(dtype, int(trans_a), int(trans_b), M, N, K, _ptr(A), _ptr(B), _ptr(bias), _ptr(Cout),
                            int(out_f32_accumulate), _ptr(ws), ws_bytes, _stream(stream)))


def dh_layernorm_fwd(dtype, T, H, x, residual, residual_bias, gamma, beta, eps, x_out, h, mu, rstd, stream=None):
    _check(lib.dh_layernorm_fwd(dtype, T, H, _ptr(x), _ptr(residual), _ptr(residual_bias), _ptr(gamma), _ptr(beta), eps,
                                _ptr(x_out), _ptr(h), _ptr(mu), _ptr(rstd), _stream(stream)))


def dh_layernorm_bwd_ws_bytes(T, H):
    return lib.dh_layernorm_bwd_ws_bytes(T, H)


def dh_layernorm_bwd(dtype, T, H, dy, x, gamma, mu, rstd, dres, dx, dgamma, dbeta, ws, ws_bytes, stream=None):
    _check(lib.dh_layernorm_bwd(dtype, T, H, _ptr(dy), _ptr(x), _ptr(gamma), _ptr(mu), _ptr(rstd), _ptr(dres), _ptr(dx),
                                _ptr(dgamma), _ptr(dbeta), _ptr(ws), ws_bytes, _stream(stream)))


def dh_rope_pairs(dtype, pairing, T, seq, pos0, n_heads, head_dim, row_stride, base, inverse, t, stream=None):
    _check(lib.dh_rope_pairs(dtype, pairing, T, seq, pos0, n_heads, head_dim, row_stride, base, int(inverse), _ptr(t),
                             _stream(stream)))


def dh_gelu_fwd_form(dtype, form, n, f, a, stream=None):
    _check(lib.dh_gelu_fwd_form(dtype, form, n, _ptr(f), _ptr(a), _stream(stream)))


def dh_gelu_bwd_form(dtype, form, n, f, da, df, stream=None):
    _check(lib.dh_gelu_bwd_form(dtype, form, n, _ptr(f), _ptr(da), _ptr(df), _stream(stream)))


def dh_gelu_fwd(dtype, n, f, a, stream=None):
    _check(lib.dh_gelu_fwd(dtype, n, _ptr(f), _ptr(a), _stream(stream)))


def dh_gelu_bwd(dtype, n, f, da, df, stream=None):
    _check(lib.dh_gelu_bwd(dtype, n, _ptr(f), _ptr(da), _ptr(df), _stream(stream)))


def dh_bias_residual_add(dtype, T, H, a, b, bias, out, stream=None):
    _check(lib.dh_bias_residual_add(dtype, T, H, _ptr(a), _ptr(b), _ptr(bias), _ptr(out), _stream(stream)))


def dh_colsum_ws_bytes(T, N):
    return lib.dh_colsum_ws_bytes(T, N)


def dh_colsum(dtype, T, N, x, out, ws, ws_bytes, stream=None):
    _check(lib.dh_colsum(dtype, T, N, _ptr(x), _ptr(out), _ptr(ws), ws_bytes, _stream(stream)))


FWD_OPS = op_names(DH_ARCH_LLAMA, 0)
BWD_OPS = op_names(DH_ARCH_LLAMA, 1)
