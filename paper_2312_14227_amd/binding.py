"""ctypes binding of libet.so: same names and arguments as include/et.h.

Only marshalling happens here: pointers are taken from integers (device addresses, e.g.
torch.Tensor.data_ptr()) or numpy arrays (host memory); every computation runs in the library.
"""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  (first: libet.so must bind to the HIP runtime torch has already loaded, so
#                            that the device pointers torch hands out and our launches share one runtime)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libet.so")

ET_OK, ET_INFEASIBLE, ET_EINVAL, ET_ENOMEM, ET_EHIP, ET_ENAN, ET_ESTATE = 0, 1, -1, -2, -3, -4, -5
ET_MLP, ET_VIT, ET_RESNET, ET_VGG, ET_MOBILENET = 0, 1, 2, 3, 4
ET_F32, ET_BF16 = 0, 1
ET_ADAM, ET_SGDW = 0, 1
ET_MAX_MLP_LAYERS = 16
ET_MAX_STAGES = 8


class et_model_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32), ("batch", C.c_int32), ("n_layers", C.c_int32),
                ("dims", C.c_int32 * (ET_MAX_MLP_LAYERS + 1)),
                ("tokens", C.c_int32), ("patch_dim", C.c_int32), ("width", C.c_int32), ("heads", C.c_int32),
                ("mlp", C.c_int32), ("blocks", C.c_int32), ("classes", C.c_int32), ("ln_eps", C.c_float),
                ("image", C.c_int32), ("in_ch", C.c_int32), ("stem", C.c_int32), ("n_stages", C.c_int32),
                ("stage_blocks", C.c_int32 * ET_MAX_STAGES), ("planes", C.c_int32 * ET_MAX_STAGES),
                ("expand", C.c_int32 * ET_MAX_STAGES), ("strides", C.c_int32 * ET_MAX_STAGES), ("last", C.c_int32)]


class et_opt(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("momentum", C.c_float), ("wd", C.c_float), ("step", C.c_uint64)]


class EtError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, strerror(status), status))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libet.so is not built: run `python -m paper_2312_14227_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, u64 = C.c_void_p, C.c_int32, C.c_uint64
    sig = {
        "et_create": (C.c_int, [C.POINTER(et_model_desc), vp, C.POINTER(vp)]),
        "et_destroy": (C.c_int, [vp]),
        "et_num_tensors": (C.c_int, [vp, C.POINTER(i32)]),
        "et_tensor_info": (C.c_int, [vp, i32, C.POINTER(C.c_size_t), C.POINTER(i32), C.POINTER(C.c_char_p)]),
        "et_workspace_bytes": (C.c_size_t, [vp]),
        "et_state_slots": (C.c_int, [vp, C.POINTER(i32)]),
        "et_bind": (C.c_int, [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), vp, C.c_size_t]),
        "et_profile": (C.c_int, [vp, vp, vp, i32, i32, C.POINTER(u64), C.POINTER(u64), C.POINTER(u64)]),
        "et_importance": (C.c_int, [vp, vp, vp, C.POINTER(vp), C.POINTER(C.c_double)]),
        "et_importance_master": (C.c_int, [vp, vp, vp, C.POINTER(vp), C.POINTER(C.c_double)]),
        "et_select": (C.c_int, [i32, C.POINTER(C.c_double), C.POINTER(u64), C.POINTER(u64), u64, C.c_uint32,
                                C.c_uint32, C.POINTER(C.c_uint8), C.POINTER(u64)]),
        "et_train_step": (C.c_int, [vp, vp, vp, C.POINTER(C.c_uint8), C.POINTER(et_opt), C.POINTER(C.c_float)]),
        "et_last_launch_counts": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]),
        "et_kernel_timing": (C.c_int, [vp, i32]),
        "et_kernel_timing_read": (C.c_int, [vp, i32, C.POINTER(u64), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "et_kernel_timing_overhead": (C.c_int, [vp, C.POINTER(C.c_double)]),
        "et_last_hip_error": (C.c_char_p, [vp]),
        "et_strerror": (C.c_char_p, [C.c_int]),
        "et_debug_copy": (C.c_int, [vp, vp, C.c_size_t, vp]),
        "et_debug_mfma_peak": (C.c_int, [vp, C.c_int, C.c_int, vp]),
        "et_debug_activation": (C.c_int, [vp, C.c_char_p, C.POINTER(vp), C.POINTER(C.c_size_t)]),
        "et_debug_depthwise3x3_ws_floats": (C.c_size_t, [C.c_int] * 5),
        "et_debug_depthwise3x3": (C.c_int, [C.c_int] + [vp] * 7 + [C.c_int] * 5 + [vp]),
        "et_debug_attention": (C.c_int, [C.c_int] + [vp] * 5 + [C.c_int] * 3 + [vp]),
        "et_debug_conv3x3_split": (C.c_int, [vp, vp, vp, vp] + [C.c_int] * 5 + [vp, vp, vp, C.c_int, C.c_int, vp, C.c_int, vp]),
        "et_debug_conv3x3_dw": (C.c_int, [vp, vp, vp] + [C.c_int] * 6 + [vp, C.c_int, vp]),
        "et_debug_conv_gathered": (C.c_int, [C.c_int, vp, vp, vp] + [C.c_int] * 8 + [vp, C.c_int, vp]),
        "et_debug_stem_ws_bytes": (C.c_size_t, [C.c_int] * 5),
        "et_debug_stem": (C.c_int, [C.c_int, vp, vp, vp, vp] + [C.c_int] * 5 + [vp]),
        "et_debug_conv3x3": (C.c_int, [vp, vp, vp] + [C.c_int] * 5 + [vp, vp, C.c_int, C.c_int, vp]),
        "et_debug_gemm_bf16": (C.c_int, [vp, vp, vp] + [C.c_int] * 9 + [C.c_float, vp, vp, C.c_int, vp, C.c_int, C.c_int, vp, vp]),
    }
    for name, (res, args) in sig.items():
        f = getattr(lib, name)
        f.restype, f.argtypes = res, args
    return lib


_lib = _load()
EXPORTS = ["et_create", "et_destroy", "et_num_tensors", "et_tensor_info", "et_workspace_bytes", "et_state_slots",
           "et_bind", "et_profile", "et_importance", "et_importance_master", "et_importance_reduce_static", "et_select", "et_select_stats", "et_tensor_metric", "et_train_step", "et_last_launch_counts",
           "et_kernel_timing", "et_kernel_timing_read", "et_kernel_timing_overhead", "et_last_hip_error", "et_strerror", "et_debug_gemm_bf16", "et_debug_copy", "et_debug_mfma_peak", "et_debug_conv3x3",
           "et_debug_conv3x3_dw", "et_debug_depthwise3x3", "et_debug_depthwise3x3_ws_floats",
           "et_debug_activation", "et_debug_conv3x3_split", "et_debug_attention",
           "et_debug_conv_gathered", "et_debug_stem", "et_debug_stem_ws_bytes"]


def strerror(status):
    return _lib.et_strerror(int(status)).decode()


def et_last_hip_error(ctx):
    return _lib.et_last_hip_error(ctx).decode()


def _check(status, where, allow=(), ctx=None):
    if status != ET_OK and status not in allow:
        if status == ET_EHIP and ctx is not None:
            where = "%s [%s]" % (where, et_last_hip_error(ctx))
        raise EtError(status, where)
    return status


def _ptr_array(ptrs):
    arr = (C.c_void_p * len(ptrs))()
    for i, p in enumerate(ptrs):
        arr[i] = p
    return arr


def make_desc(kind, dtype, batch, dims=(), tokens=0, patch_dim=0, width=0, heads=0, mlp=0, blocks=0, classes=0,
              ln_eps=1e-6, image=0, in_ch=0, stem=0, stage_blocks=(), planes=(), expand=(), strides=(), last=0):
    d = et_model_desc()
    d.kind, d.dtype, d.batch = kind, dtype, batch
    d.n_layers = max(len(dims) - 1, 0)
    for i, v in enumerate(dims):
        d.dims[i] = v
    d.tokens, d.patch_dim, d.width, d.heads, d.mlp, d.blocks, d.classes = tokens, patch_dim, width, heads, mlp, blocks, classes
    d.ln_eps = ln_eps
    d.image, d.in_ch, d.stem, d.n_stages = image, in_ch, stem, len(stage_blocks)
    for i, (nb, pl) in enumerate(zip(stage_blocks, planes)):
        d.stage_blocks[i], d.planes[i] = nb, pl
    for i, (e, st) in enumerate(zip(expand, strides)):
        d.expand[i], d.strides[i] = e, st
    d.last = last
    return d


def et_create(desc, hip_stream=0):
    out = C.c_void_p()
    _check(_lib.et_create(C.byref(desc), C.c_void_p(hip_stream), C.byref(out)), "et_create")
    return out


def et_destroy(ctx):
    _check(_lib.et_destroy(ctx), "et_destroy")


def et_num_tensors(ctx):
    n = C.c_int32()
    _check(_lib.et_num_tensors(ctx, C.byref(n)), "et_num_tensors")
    return n.value


def et_tensor_info(ctx, i):
    numel, dtype, name = C.c_size_t(), C.c_int32(), C.c_char_p()
    _check(_lib.et_tensor_info(ctx, i, C.byref(numel), C.byref(dtype), C.byref(name)), "et_tensor_info")
    return numel.value, dtype.value, name.value.decode()


def et_workspace_bytes(ctx):
    return _lib.et_workspace_bytes(ctx)


def et_state_slots(ctx):
    k = C.c_int32()
    _check(_lib.et_state_slots(ctx, C.byref(k)), "et_state_slots")
    return k.value


def et_bind(ctx, w_dev, opt_state_dev, grad_dev, workspace_dev, workspace_bytes):
    st = _ptr_array(opt_state_dev) if opt_state_dev is not None else None
    _check(_lib.et_bind(ctx, _ptr_array(w_dev), st, _ptr_array(grad_dev), C.c_void_p(workspace_dev), workspace_bytes),
           "et_bind", ctx=ctx)


def et_profile(ctx, x_dev, y_dev, warmup, reps):
    n = et_num_tensors(ctx)
    t_fwd = C.c_uint64()
    t_dw, t_dy = (C.c_uint64 * n)(), (C.c_uint64 * n)()
    _check(_lib.et_profile(ctx, C.c_void_p(x_dev), C.c_void_p(y_dev), warmup, reps, C.byref(t_fwd), t_dw, t_dy),
           "et_profile", ctx=ctx)
    return t_fwd.value, np.array(t_dw[:], dtype=np.uint64), np.array(t_dy[:], dtype=np.uint64)


def et_importance(ctx, x_dev, y_dev, w_snapshot_dev):
    n = et_num_tensors(ctx)
    out = (C.c_double * n)()
    _check(_lib.et_importance(ctx, C.c_void_p(x_dev), C.c_void_p(y_dev), _ptr_array(w_snapshot_dev), out),
           "et_importance", ctx=ctx)
    return np.array(out[:], dtype=np.float64)


def et_importance_master(ctx, x_dev, y_dev, w_snapshot_f32_dev):
    n = et_num_tensors(ctx)
    out = (C.c_double * n)()
    _check(_lib.et_importance_master(ctx, C.c_void_p(x_dev), C.c_void_p(y_dev), _ptr_array(w_snapshot_f32_dev), out),
           "et_importance_master", ctx=ctx)
    return np.array(out[:], dtype=np.float64)


def et_importance_reduce_static(grad_dev, w_dev, w_snapshot_dev, numel, dtype, stream, importance_dev):
    """Enqueues the allocation-free Eq. 2 reduction; importance_dev is a device address of len(numel) doubles."""
    n = len(numel)
    sizes = (C.c_uint64 * max(n, 1))(*[int(v) for v in numel])
    _check(_lib.et_importance_reduce_static(C.c_int32(n), _ptr_array(grad_dev), _ptr_array(w_dev), _ptr_array(w_snapshot_dev),
                                            sizes, C.c_int32(dtype), C.c_void_p(stream), C.c_void_p(importance_dev)),
           "et_importance_reduce_static")


def et_select(importance, t_dw_ns, t_dy_ns, t_fwd_ns, rho_ppm, tq):
    """Returns (status, mask uint8[N], predicted_ns); raises on errors other than ET_INFEASIBLE."""
    imp = np.ascontiguousarray(importance, dtype=np.float64)
    dw = np.ascontiguousarray(t_dw_ns, dtype=np.uint64)
    dy = np.ascontiguousarray(t_dy_ns, dtype=np.uint64)
    n = imp.size
    mask = np.zeros(max(n, 1), dtype=np.uint8)
    pred = C.c_uint64()
    st = _lib.et_select(n, imp.ctypes.data_as(C.POINTER(C.c_double)), dw.ctypes.data_as(C.POINTER(C.c_uint64)),
                        dy.ctypes.data_as(C.POINTER(C.c_uint64)), int(t_fwd_ns), int(rho_ppm), int(tq),
                        mask.ctypes.data_as(C.POINTER(C.c_uint8)), C.byref(pred))
    _check(st, "et_select", allow=(ET_INFEASIBLE,))
    return st, mask[:n].copy(), pred.value


ET_METRIC_WEIGHT_L1, ET_METRIC_GRAD_L1 = 1, 2


def et_tensor_metric(ctx, x_dev, y_dev, metric, n):
    out = (C.c_double * n)()
    _lib.et_tensor_metric.restype = C.c_int
    _check(_lib.et_tensor_metric(ctx, C.c_void_p(x_dev), C.c_void_p(y_dev), C.c_int32(metric), out), "et_tensor_metric", ctx=ctx)
    return np.array(out[:], dtype=np.float64)


class et_select_counts(C.Structure):
    _fields_ = [("backward_q", C.c_uint64), ("budget_q", C.c_uint64), ("cells_table", C.c_uint64),
                ("cells_pruned", C.c_uint64), ("cells_knapsack", C.c_uint64)]


def et_select_stats(importance, t_dw_ns, t_dy_ns, t_fwd_ns, rho_ppm, tq):
    """Returns (status, mask uint8[N], predicted_ns, counts dict)."""
    imp = np.ascontiguousarray(importance, dtype=np.float64)
    dw = np.ascontiguousarray(t_dw_ns, dtype=np.uint64)
    dy = np.ascontiguousarray(t_dy_ns, dtype=np.uint64)
    n = imp.size
    mask = np.zeros(max(n, 1), dtype=np.uint8)
    pred = C.c_uint64()
    cnt = et_select_counts()
    _lib.et_select_stats.restype = C.c_int
    st = _lib.et_select_stats(C.c_int32(n), imp.ctypes.data_as(C.POINTER(C.c_double)), dw.ctypes.data_as(C.POINTER(C.c_uint64)),
                              dy.ctypes.data_as(C.POINTER(C.c_uint64)), C.c_uint64(int(t_fwd_ns)), C.c_uint32(int(rho_ppm)),
                              C.c_uint32(int(tq)), mask.ctypes.data_as(C.POINTER(C.c_uint8)), C.byref(pred), C.byref(cnt))
    _check(st, "et_select_stats", allow=(ET_INFEASIBLE,))
    return st, mask[:n].copy(), pred.value, {k: int(getattr(cnt, k)) for k, _ in et_select_counts._fields_}


def et_train_step(ctx, x_dev, y_dev, mask, opt=None, want_loss=True):
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    loss = C.c_float()
    _check(_lib.et_train_step(ctx, C.c_void_p(x_dev), C.c_void_p(y_dev), m.ctypes.data_as(C.POINTER(C.c_uint8)),
                              C.byref(opt) if opt is not None else None, C.byref(loss) if want_loss else None),
           "et_train_step", ctx=ctx)
    return loss.value if want_loss else None


def et_last_launch_counts(ctx):
    f, b, u = C.c_int32(), C.c_int32(), C.c_int32()
    _check(_lib.et_last_launch_counts(ctx, C.byref(f), C.byref(b), C.byref(u)), "et_last_launch_counts")
    return f.value, b.value, u.value


def et_kernel_timing(ctx, enable):
    _check(_lib.et_kernel_timing(ctx, int(enable)), "et_kernel_timing", ctx=ctx)


def et_kernel_timing_overhead(ctx):
    """Median elapsed time (ns) of an event pair with nothing between its events, measured when timing was enabled."""
    ns = C.c_double(0.0)
    _check(_lib.et_kernel_timing_overhead(ctx, C.byref(ns)), "et_kernel_timing_overhead", ctx=ctx)
    return ns.value


def et_kernel_timing_read(ctx, kernel_class):
    """(launches, total_ns, work) of one kernel class since timing was enabled."""
    n, ns, w = C.c_uint64(), C.c_double(), C.c_double()
    _check(_lib.et_kernel_timing_read(ctx, kernel_class, C.byref(n), C.byref(ns), C.byref(w)), "et_kernel_timing_read", ctx=ctx)
    return n.value, ns.value, w.value


def et_debug_gemm_bf16(A, B, Cp, M, N, K, lda, ldb, ldc, a_t, b_t, c_f32, alpha=1.0, bias=0, residual=0, split_k=1,
                       partials=0, tile=0, stream=0, epilogue=0, aux=0):
    return _lib.et_debug_gemm_bf16(C.c_void_p(A), C.c_void_p(B), C.c_void_p(Cp), M, N, K, lda, ldb, ldc, int(a_t),
                                   int(b_t), int(c_f32), alpha, C.c_void_p(bias), C.c_void_p(residual), split_k,
                                   C.c_void_p(partials), tile, int(epilogue), C.c_void_p(aux), C.c_void_p(stream))


def et_debug_conv3x3(x, w, out, batch, H, W, Cin, N, bias=0, U=0, mode=0, tile=0, stream=0):
    return _lib.et_debug_conv3x3(C.c_void_p(x), C.c_void_p(w), C.c_void_p(out), batch, H, W, Cin, N, C.c_void_p(bias),
                                 C.c_void_p(U), mode, tile, C.c_void_p(stream))


def et_debug_conv3x3_split(x, w, out, z_out, batch, H, W, Cin, N, bias=0, gain=0, U=0, mode=0, split_k=0, partials=0, tile=0,
                           stream=0):
    return _lib.et_debug_conv3x3_split(C.c_void_p(x), C.c_void_p(w), C.c_void_p(out), C.c_void_p(z_out), batch, H, W, Cin, N,
                                       C.c_void_p(bias), C.c_void_p(gain), C.c_void_p(U), mode, split_k, C.c_void_p(partials), tile,
                                       C.c_void_p(stream))


def et_debug_conv3x3_dw(x, d, dw, batch, H, W, Cin, N, split_k=1, partials=0, tile=0, stream=0):
    return _lib.et_debug_conv3x3_dw(C.c_void_p(x), C.c_void_p(d), C.c_void_p(dw), batch, H, W, Cin, N, split_k,
                                    C.c_void_p(partials), tile, C.c_void_p(stream))


def et_debug_conv_gathered(op, x, w_or_d, out, batch, H, W, Cin, N, taps=3, stride=1, split_k=1, partials=0, tile=0, stream=0):
    return _lib.et_debug_conv_gathered(op, C.c_void_p(x), C.c_void_p(w_or_d), C.c_void_p(out), batch, H, W, Cin, N, taps, stride,
                                       split_k, C.c_void_p(partials), tile, C.c_void_p(stream))


def et_debug_stem_ws_bytes(batch, H, W, Cin, N):
    return int(_lib.et_debug_stem_ws_bytes(batch, H, W, Cin, N))


def et_debug_stem(op, x, w_or_d, out, ws, batch, H, W, Cin, N, stream=0):
    return _lib.et_debug_stem(op, C.c_void_p(x), C.c_void_p(w_or_d), C.c_void_p(out), C.c_void_p(ws), batch, H, W, Cin, N,
                              C.c_void_p(stream))


def et_debug_activation(ctx, name):
    """(device address, element count) of a stored bf16 activation."""
    p, n = C.c_void_p(), C.c_size_t()
    _check(_lib.et_debug_activation(ctx, name.encode(), C.byref(p), C.byref(n)), "et_debug_activation")
    return p.value, n.value


def et_debug_depthwise3x3(op, a, b, gain, shift, out0, out1, ws, batch, H, W, Cch, stride, stream=0):
    return _lib.et_debug_depthwise3x3(op, C.c_void_p(a), C.c_void_p(b), C.c_void_p(gain), C.c_void_p(shift), C.c_void_p(out0),
                                      C.c_void_p(out1), C.c_void_p(ws), batch, H, W, Cch, stride, C.c_void_p(stream))


def et_debug_depthwise3x3_ws_floats(batch, H, W, Cch, stride):
    return _lib.et_debug_depthwise3x3_ws_floats(batch, H, W, Cch, stride)


def et_debug_attention(op, qkv, out, lse, dout, dqkv, B, T, H, stream=0):
    return _lib.et_debug_attention(op, C.c_void_p(qkv), C.c_void_p(out), C.c_void_p(lse), C.c_void_p(dout), C.c_void_p(dqkv),
                                   B, T, H, C.c_void_p(stream))


def et_debug_mfma_peak(out, workgroups, iters, stream=0):
    return _lib.et_debug_mfma_peak(C.c_void_p(out), workgroups, iters, C.c_void_p(stream))


def et_debug_copy(dst, src, nbytes, stream=0):
    return _lib.et_debug_copy(C.c_void_p(dst), C.c_void_p(src), nbytes, C.c_void_p(stream))
