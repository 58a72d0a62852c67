"""Thin ctypes binding over libjpp.so: same names as include/jpp.h, argument marshalling
only.  Every computation happens inside the library's HIP kernels; there is no fallback.
If the library has not been built, loading raises (build with
`python -m paper_2412_14374_amd.build`)."""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libjpp.so")

JPP_OK, JPP_EINVAL, JPP_ESCHED, JPP_ECAPACITY, JPP_EDEVICE, JPP_ESTATE = range(6)
JPP_FWD, JPP_BWD = 0, 1
JPP_F32, JPP_BF16 = 0, 1
JPP_MAX_VIRTUAL = 8
OUT_STORE, OUT_STORE_F32, OUT_ACC_F32 = 0, 1, 2


class JppError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"jpp status {status}: {message}")
        self.status = status


class jpp_task(C.Structure):
    _fields_ = [("i", C.c_int32), ("ty", C.c_int32), ("stage", C.c_int32)]


class jpp_layer_config(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("n_layers", C.c_int32), ("d_model", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ffn", C.c_int32), ("seq_len", C.c_int32), ("microbatch", C.c_int32),
                ("norm", C.c_int32), ("act", C.c_int32), ("use_bias", C.c_int32), ("rope", C.c_int32),
                ("rope_theta", C.c_float), ("norm_eps", C.c_float), ("loss_head", C.c_int32),
                ("vocab", C.c_int32), ("remat", C.c_int32), ("wgrad_group", C.c_int32), ("embed", C.c_int32), ("n_virtual", C.c_int32), ("stage_ids", C.c_int32 * JPP_MAX_VIRTUAL)]


class jpp_optimizer_step(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("step", C.c_int32)]


JPP_OPT_SGD, JPP_OPT_ADAMW = 0, 1

_lib = None

_SIGNATURES = {
    "jpp_schedule_len": (C.c_int, [C.c_int] * 5),
    "jpp_schedule_make": (C.c_int, [C.c_int] * 5 + [C.POINTER(jpp_task), C.c_int]),
    "jpp_schedule_validate": (C.c_int, [C.POINTER(jpp_layer_config), C.c_int, C.POINTER(jpp_task), C.c_int,
                                        C.POINTER(C.c_int)]),
    "jpp_stage_arena_bytes": (C.c_size_t, [C.POINTER(jpp_layer_config), C.c_int, C.c_int]),
    "jpp_stage_create": (C.c_int, [C.POINTER(jpp_layer_config), C.c_int, C.c_int, C.c_void_p, C.c_size_t,
                                   C.POINTER(C.c_void_p)]),
    "jpp_stage_destroy": (None, [C.c_void_p]),
    "jpp_stage_param_info": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_int64),
                                       C.POINTER(C.c_size_t)]),
    "jpp_stage_param_count": (C.c_size_t, [C.c_void_p]),
    "jpp_stage_set_params": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int]),
    "jpp_stage_bind_boundary": (C.c_int, [C.c_void_p] + [C.POINTER(C.c_void_p)] * 5),
    "jpp_stage_zero_grads": (C.c_int, [C.c_void_p, C.c_void_p]),
    "jpp_stage_run": (C.c_int, [C.c_void_p, C.POINTER(jpp_task), C.c_int, C.c_void_p, C.c_void_p]),
    "jpp_stage_grads": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_void_p), C.POINTER(C.c_size_t)]),
    "jpp_stage_losses": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p)]),
    "jpp_pipeline_merge_order": (C.c_int, [C.c_int] * 3 + [C.POINTER(C.POINTER(jpp_task)), C.POINTER(C.c_int),
                                                           C.POINTER(C.c_int), C.c_int]),
    "jpp_pipeline_arena_bytes": (C.c_size_t, [C.POINTER(jpp_layer_config), C.c_int, C.c_int]),
    "jpp_pipeline_create": (C.c_int, [C.POINTER(C.c_void_p), C.c_int, C.c_void_p, C.c_size_t,
                                      C.POINTER(C.c_void_p)]),
    "jpp_pipeline_destroy": (None, [C.c_void_p]),
    "jpp_pipeline_bind": (C.c_int, [C.c_void_p] + [C.POINTER(C.c_void_p)] * 5),
    "jpp_pipeline_run": (C.c_int, [C.c_void_p, C.POINTER(C.POINTER(jpp_task)), C.POINTER(C.c_int),
                                   C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]),
    "jpp_pipeline_sync": (C.c_int, [C.c_void_p]),
    "jpp_pipeline_sum_tied_gradients": (C.c_int, [C.c_void_p, C.c_void_p]),
    "jpp_stage_params": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_void_p), C.POINTER(C.c_size_t)]),
    "jpp_stage_optimizer_bytes": (C.c_size_t, [C.c_void_p, C.c_int]),
    "jpp_stage_optimizer_bind": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "jpp_stage_apply_gradients": (C.c_int, [C.c_void_p, C.POINTER(jpp_optimizer_step), C.c_void_p]),
    "jpp_stage_peak_in_flight": (C.c_int, [C.c_void_p]),
    "jpp_stage_pending_peak": (C.c_int, [C.c_void_p]),
    "jpp_stage_prefetched": (C.c_int, [C.c_void_p]),
    "jpp_last_error": (C.c_char_p, []),
    "jpp_set_gemm_variant": (None, [C.c_int]),
    "jpp_set_stream_mode": (None, [C.c_int]),
    "jpp_set_fused_activation": (None, [C.c_int]),
    "jpp_stage_stream_mode": (C.c_int, [C.c_void_p]),
    "jpp_op_gemm_workspace_bytes": (C.c_size_t, [C.c_int] * 5),
    "jpp_op_gemm_ws": (C.c_int, [C.c_int] * 4 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                  C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                                  C.c_void_p, C.c_size_t, C.c_void_p]),
    "jpp_op_gemm": (C.c_int, [C.c_int] * 4 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                              C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "jpp_op_gemm_gelu": (C.c_int, [C.c_int] * 3 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                   C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                   C.c_size_t, C.c_void_p]),
    "jpp_op_attention_fwd": (C.c_int, [C.c_int] * 6 + [C.c_void_p] * 4),
    "jpp_op_attention_bwd": (C.c_int, [C.c_int] * 6 + [C.c_void_p] * 7),
    "jpp_op_norm_fwd": (C.c_int, [C.c_int] * 4 + [C.c_float] + [C.c_void_p] * 6),
    "jpp_op_norm_bwd": (C.c_int, [C.c_int] * 4 + [C.c_void_p] * 10),
    "jpp_op_colreduce_scratch": (C.c_size_t, [C.c_int, C.c_int]),
    "jpp_op_act_fwd": (C.c_int, [C.c_int] * 4 + [C.c_void_p] * 3),
    "jpp_op_act_bwd": (C.c_int, [C.c_int] * 4 + [C.c_void_p] * 4),
    "jpp_op_cross_entropy": (C.c_int, [C.c_int] * 3 + [C.c_void_p] * 6),
    "jpp_op_attention_bwd_scratch_bytes": (C.c_size_t, [C.c_int] * 6),
    "jpp_op_attention_bwd_ws": (C.c_int, [C.c_int] * 6 + [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p]),
    "jpp_op_attention_bwd_static": (C.c_int, [C.c_int] * 6 + [C.c_void_p] * 6),
    "jpp_op_embed_fwd": (C.c_int, [C.c_int] * 4 + [C.c_void_p] * 4),
    "jpp_op_embed_bwd": (C.c_int, [C.c_int] * 4 + [C.c_void_p] * 4),
}


def lib():
    """Loads libjpp.so once.  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2412_14374_amd.build`")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def exported_names():
    return sorted(_SIGNATURES)


def last_error():
    return lib().jpp_last_error().decode()


def _check(status):
    if status != JPP_OK:
        raise JppError(status, last_error())


def make_config(w):
    """w: any object with the jpp_layer_config field names as attributes plus `stage_ids`."""
    c = jpp_layer_config()
    for f, _ in jpp_layer_config._fields_:
        if f in ("stage_ids", "n_virtual"):
            continue
        optional = f in ("remat", "wgrad_group", "embed")
        setattr(c, f, getattr(w, f, 0) if optional else getattr(w, f))
    ids = list(w.stage_ids)
    c.n_virtual = len(ids)
    for k, s in enumerate(ids):
        c.stage_ids[k] = s
    return c


def tasks_array(tasks):
    """tasks: iterable of (i, ty, stage) with ty 0/1 or 'fwd'/'bwd'."""
    tasks = list(tasks)
    arr = (jpp_task * max(1, len(tasks)))()
    for k, (i, ty, s) in enumerate(tasks):
        arr[k].i = i
        arr[k].ty = {"fwd": JPP_FWD, "bwd": JPP_BWD}.get(ty, ty)
        arr[k].stage = s
    return arr, len(tasks)


def jpp_schedule_len(kind, P, rank, V, M):
    return lib().jpp_schedule_len(kind, P, rank, V, M)


def jpp_schedule_make(kind, P, rank, V, M):
    n = jpp_schedule_len(kind, P, rank, V, M)
    if n < 0:
        raise JppError(JPP_EINVAL, "bad schedule arguments")
    arr = (jpp_task * n)()
    _check(lib().jpp_schedule_make(kind, P, rank, V, M, arr, n))
    return [(t.i, t.ty, t.stage) for t in arr]


def jpp_schedule_validate(cfg, M, tasks):
    arr, n = tasks_array(tasks)
    peak = C.c_int(0)
    _check(lib().jpp_schedule_validate(C.byref(cfg), M, arr, n, C.byref(peak)))
    return peak.value


def jpp_stage_arena_bytes(cfg, M, max_in_flight):
    n = lib().jpp_stage_arena_bytes(C.byref(cfg), M, max_in_flight)
    if n == 0:
        raise JppError(JPP_EINVAL, last_error())
    return n


def jpp_stage_create(cfg, M, max_in_flight, arena_ptr, arena_bytes):
    h = C.c_void_p()
    _check(lib().jpp_stage_create(C.byref(cfg), M, max_in_flight, C.c_void_p(arena_ptr), arena_bytes, C.byref(h)))
    return h


def jpp_stage_destroy(h):
    lib().jpp_stage_destroy(h)


def jpp_stage_param_info(h):
    """Returns [(name, shape tuple, element offset)]."""
    n = lib().jpp_stage_param_info(h, -1, None, None, None)
    if n < 0:
        raise JppError(-n, last_error())
    out = []
    for k in range(n):
        name = C.c_char_p()
        shape = (C.c_int64 * 2)()
        off = C.c_size_t()
        _check(lib().jpp_stage_param_info(h, k, C.byref(name), shape, C.byref(off)))
        shp = (shape[0],) if shape[1] == 0 else (shape[0], shape[1])
        out.append((name.value.decode(), shp, off.value))
    return out


def jpp_stage_param_count(h):
    return lib().jpp_stage_param_count(h)


def jpp_stage_set_params(h, vstage, ptr, on_device):
    _check(lib().jpp_stage_set_params(h, vstage, C.c_void_p(ptr), 1 if on_device else 0))


def _ptr_array(ptrs):
    if ptrs is None:
        return None
    arr = (C.c_void_p * len(ptrs))()
    for k, p in enumerate(ptrs):
        arr[k] = p
    return arr


def jpp_stage_bind_boundary(h, inbox_x, inbox_cot, outbox_y, outbox_dx, targets):
    """Each argument: list of device addresses (ints), indexed [vstage*M + i], or None."""
    _check(lib().jpp_stage_bind_boundary(h, _ptr_array(inbox_x), _ptr_array(inbox_cot), _ptr_array(outbox_y),
                                         _ptr_array(outbox_dx), _ptr_array(targets)))


def jpp_stage_zero_grads(h, stream):
    _check(lib().jpp_stage_zero_grads(h, C.c_void_p(stream)))


def jpp_stage_run(h, tasks_arr, n, compute_stream, side_stream):
    _check(lib().jpp_stage_run(h, tasks_arr, n, C.c_void_p(compute_stream), C.c_void_p(side_stream)))


def jpp_stage_grads(h, vstage):
    p = C.c_void_p()
    n = C.c_size_t()
    _check(lib().jpp_stage_grads(h, vstage, C.byref(p), C.byref(n)))
    return p.value, n.value


def jpp_stage_losses(h):
    p = C.c_void_p()
    _check(lib().jpp_stage_losses(h, C.byref(p)))
    return p.value


def jpp_pipeline_merge_order(P, V, M, task_lists):
    """Returns [actor, ...]: which actor enqueues its next task at each step."""
    arrs = [tasks_array(t) for t in task_lists]
    lists = (C.POINTER(jpp_task) * P)(*[C.cast(a, C.POINTER(jpp_task)) for a, _ in arrs])
    counts = (C.c_int * P)(*[n for _, n in arrs])
    total = sum(n for _, n in arrs)
    out = (C.c_int * max(total, 1))()
    _check(lib().jpp_pipeline_merge_order(P, V, M, lists, counts, out, total))
    return list(out[:total])


def jpp_pipeline_arena_bytes(cfg, n_actors, M):
    return lib().jpp_pipeline_arena_bytes(C.byref(cfg), n_actors, M)


def jpp_pipeline_create(actor_handles, arena_ptr, arena_bytes):
    h = C.c_void_p()
    arr = (C.c_void_p * len(actor_handles))(*[a.value if hasattr(a, "value") else a for a in actor_handles])
    _check(lib().jpp_pipeline_create(arr, len(actor_handles), C.c_void_p(arena_ptr), arena_bytes, C.byref(h)))
    return h


def jpp_pipeline_destroy(h):
    lib().jpp_pipeline_destroy(h)


def jpp_pipeline_bind(h, x_in, dx_out, targets, cot_in, y_out):
    """Each argument: list of M device addresses (ints) or None."""
    _check(lib().jpp_pipeline_bind(h, _ptr_array(x_in), _ptr_array(dx_out), _ptr_array(targets),
                                   _ptr_array(cot_in), _ptr_array(y_out)))


def jpp_pipeline_run(h, task_lists, compute_streams, side_streams):
    """task_lists: one list of (i, ty, stage) per actor; streams: raw stream handles (ints)."""
    P = len(task_lists)
    arrs = [tasks_array(t) for t in task_lists]
    lists = (C.POINTER(jpp_task) * P)(*[C.cast(a, C.POINTER(jpp_task)) for a, _ in arrs])
    counts = (C.c_int * P)(*[n for _, n in arrs])
    _check(lib().jpp_pipeline_run(h, lists, counts, _ptr_array(compute_streams), _ptr_array(side_streams)))


def jpp_pipeline_sync(h):
    _check(lib().jpp_pipeline_sync(h))


def jpp_pipeline_sum_tied_gradients(h, stream):
    _check(lib().jpp_pipeline_sum_tied_gradients(h, C.c_void_p(stream)))


def jpp_stage_params(h, vstage):
    p = C.c_void_p()
    n = C.c_size_t()
    _check(lib().jpp_stage_params(h, vstage, C.byref(p), C.byref(n)))
    return p.value, n.value


def jpp_stage_optimizer_bytes(h, kind):
    return lib().jpp_stage_optimizer_bytes(h, kind)


def jpp_stage_optimizer_bind(h, kind, state_ptr, state_bytes, stream):
    _check(lib().jpp_stage_optimizer_bind(h, kind, C.c_void_p(state_ptr), state_bytes, C.c_void_p(stream)))


def jpp_stage_apply_gradients(h, kind, lr, stream, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, step=1):
    o = jpp_optimizer_step(kind, lr, beta1, beta2, eps, weight_decay, step)
    _check(lib().jpp_stage_apply_gradients(h, C.byref(o), C.c_void_p(stream)))


def jpp_stage_peak_in_flight(h):
    return lib().jpp_stage_peak_in_flight(h)


def jpp_stage_pending_peak(h):
    return lib().jpp_stage_pending_peak(h)


def jpp_stage_prefetched(h):
    return lib().jpp_stage_prefetched(h)


def jpp_set_stream_mode(mode):
    lib().jpp_set_stream_mode(mode)


def jpp_set_fused_activation(mask):
    lib().jpp_set_fused_activation(mask)


def jpp_stage_stream_mode(h):
    return lib().jpp_stage_stream_mode(h)


def jpp_set_gemm_variant(v):
    lib().jpp_set_gemm_variant(v)


def jpp_op_gemm(dtype, M, N, K, A, lda, a_ks, B, ldb, b_ks, Cp, ldc, out_mode, bias, residual, stream):
    _check(lib().jpp_op_gemm(dtype, M, N, K, A, lda, int(a_ks), B, ldb, int(b_ks), Cp, ldc, out_mode, bias,
                             residual, stream))


def jpp_op_gemm_workspace_bytes(dtype, M, N, K, out_mode):
    return lib().jpp_op_gemm_workspace_bytes(dtype, M, N, K, out_mode)


def jpp_op_gemm_ws(dtype, M, N, K, A, lda, a_ks, B, ldb, b_ks, Cp, ldc, out_mode, bias, residual, workspace,
                   workspace_bytes, stream):
    _check(lib().jpp_op_gemm_ws(dtype, M, N, K, A, lda, int(a_ks), B, ldb, int(b_ks), Cp, ldc, out_mode, bias,
                                residual, workspace, workspace_bytes, stream))


def jpp_op_gemm_gelu(M, N, K, A, lda, a_ks, B, ldb, b_ks, Cp, ldc, bias, act, backward, aux, workspace,
                     workspace_bytes, stream):
    _check(lib().jpp_op_gemm_gelu(M, N, K, A, lda, int(a_ks), B, ldb, int(b_ks), Cp, ldc, bias, act, int(backward), aux,
                                  workspace, workspace_bytes, stream))


def jpp_op_attention_fwd(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, stream):
    _check(lib().jpp_op_attention_fwd(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, stream))


def jpp_op_attention_bwd(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, dout, dqkv, delta, stream):
    _check(lib().jpp_op_attention_bwd(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, dout, dqkv, delta, stream))


def jpp_op_norm_fwd(dtype, norm, rows, d, eps, x, gamma, beta, y, stats, stream):
    _check(lib().jpp_op_norm_fwd(dtype, norm, rows, d, eps, x, gamma, beta, y, stats, stream))


def jpp_op_norm_bwd(dtype, norm, rows, d, x, gamma, stats, dy, dx_add, dx, g_gamma, g_beta, partial, stream):
    _check(lib().jpp_op_norm_bwd(dtype, norm, rows, d, x, gamma, stats, dy, dx_add, dx, g_gamma, g_beta, partial,
                                 stream))


def jpp_op_colreduce_scratch(rows, d):
    return lib().jpp_op_colreduce_scratch(rows, d)


def jpp_op_act_fwd(dtype, act, rows, f, h, a, stream):
    _check(lib().jpp_op_act_fwd(dtype, act, rows, f, h, a, stream))


def jpp_op_act_bwd(dtype, act, rows, f, h, da, dh, stream):
    _check(lib().jpp_op_act_bwd(dtype, act, rows, f, h, da, dh, stream))


def jpp_op_attention_bwd_scratch_bytes(dtype, mb, seq, Hq, Hkv, hd):
    return lib().jpp_op_attention_bwd_scratch_bytes(dtype, mb, seq, Hq, Hkv, hd)


def jpp_op_attention_bwd_ws(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, dout, dqkv, delta, scratch, scratch_bytes,
                            stream):
    _check(lib().jpp_op_attention_bwd_ws(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, dout, dqkv, delta, scratch,
                                         scratch_bytes, stream))


JPP_STATIC_SCRATCH_BYTES = 4 << 20


def jpp_op_attention_bwd_static(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, dout, dqkv, stream):
    _check(lib().jpp_op_attention_bwd_static(dtype, mb, seq, Hq, Hkv, hd, qkv, out, lse, dout, dqkv, stream))


def jpp_op_cross_entropy(dtype, rows, vocab, z, targets, dz, row_loss, loss, stream):
    _check(lib().jpp_op_cross_entropy(dtype, rows, vocab, z, targets, dz, row_loss, loss, stream))


def jpp_op_embed_fwd(dtype, rows, d, vocab, ids, table, x, stream):
    _check(lib().jpp_op_embed_fwd(dtype, rows, d, vocab, ids, table, x, stream))


def jpp_op_embed_bwd(dtype, rows, d, vocab, ids, dx, g_table, stream):
    _check(lib().jpp_op_embed_bwd(dtype, rows, d, vocab, ids, dx, g_table, stream))
