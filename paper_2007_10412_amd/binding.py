"""ctypes binding of librad_hip.so: same names as include/rad.h, argument
marshalling only.  Tensors are torch CUDA(HIP) tensors; every computation runs
in the library's kernels.  There is no fallback: a missing library raises."""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librad_hip.so")

RAD_OK, RAD_ERR_NULL, RAD_ERR_SHAPE, RAD_ERR_PARAM, RAD_ERR_UNSUPPORTED, RAD_ERR_CAPACITY, RAD_ERR_DEVICE = range(7)
RAD_F32, RAD_BF16 = 0, 1
(RAD_EXACT, RAD_BERNOULLI, RAD_FIXEDK_SHARED, RAD_FIXEDK_PER_EXAMPLE, RAD_REPLACE_SHARED, RAD_REPLACE_PER_EXAMPLE,
 RAD_PROJECT_SHARED, RAD_PROJECT_PER_EXAMPLE) = range(8)
RAD_LINEAR, RAD_CONV2D = 0, 1
STATUS_NAMES = ["RAD_OK", "RAD_ERR_NULL", "RAD_ERR_SHAPE", "RAD_ERR_PARAM", "RAD_ERR_UNSUPPORTED",
                "RAD_ERR_CAPACITY", "RAD_ERR_DEVICE"]


class rad_layer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32), ("batch", C.c_int64), ("d_in", C.c_int64),
                ("d_out", C.c_int64), ("relu", C.c_int32), ("has_bias", C.c_int32),
                ("c_in", C.c_int32), ("h", C.c_int32), ("w", C.c_int32), ("c_out", C.c_int32),
                ("kh", C.c_int32), ("kw", C.c_int32), ("pad", C.c_int32)]


class rad_sampling(C.Structure):
    _fields_ = [("scheme", C.c_int32), ("p", C.c_double), ("seed", C.c_uint64),
                ("stream_id", C.c_uint32), ("step", C.c_uint32)]


class rad_store_stats(C.Structure):
    _fields_ = [("value_bytes", C.c_uint64), ("index_bytes", C.c_uint64), ("bit_bytes", C.c_uint64),
                ("nnz", C.c_uint64), ("dense_bytes", C.c_uint64)]


# every symbol include/rad.h declares: name -> (restype, argtypes)
P = C.c_void_p
RAD_SGD, RAD_ADAM = 0, 1


class rad_optimizer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_double), ("l2", C.c_double), ("beta1", C.c_double),
                ("beta2", C.c_double), ("eps", C.c_double)]


class rad_pde_grid(C.Structure):
    _fields_ = [("n", C.c_int32), ("steps", C.c_int64), ("D", C.c_double), ("dt", C.c_double)]


class rad_graph(C.Structure):
    _fields_ = [("n_vertices", C.c_int32), ("n_levels", C.c_int32), ("n_edges", C.c_int64), ("level_ptr", P),
                ("succ_ptr", P), ("succ", P), ("partial", P)]


SIGNATURES = {
    "rad_fixed_k": (C.c_int64, [C.c_double, C.c_int64]),
    "rad_ctx_create": (C.c_int, [C.POINTER(P), P]),
    "rad_ctx_destroy": (C.c_int, [P]),
    "rad_last_error": (C.c_char_p, [P]),
    "rad_ctx_synchronize": (C.c_int, [P]),
    "rad_ctx_timing": (C.c_int, [P, C.c_char_p]),
    "rad_ctx_timing_read": (C.c_int, [P, C.c_char_p, C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
    "rad_ctx_timing_read_flops": (C.c_int, [P, C.c_char_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "rad_ctx_timing_reset": (C.c_int, [P]),
    "rad_debug_key_shift": (C.c_int, [P, C.c_int32]),
    "rad_probe_ceiling": (C.c_int, [P, C.c_int32, P, P, C.c_uint64, C.c_int32, C.POINTER(C.c_double)]),
    "rad_store_create": (C.c_int, [P, C.POINTER(rad_layer), C.c_int32, C.c_double, C.c_int32, C.POINTER(P)]),
    "rad_store_destroy": (C.c_int, [P]),
    "rad_store_get_stats": (C.c_int, [P, P, C.POINTER(rad_store_stats)]),
    "rad_store_export_csr": (C.c_int, [P, P, P, P, P, C.c_int64]),
    "rad_store_export_bits": (C.c_int, [P, P, P]),
    "rad_store_import_bits": (C.c_int, [P, P, P]),
    "rad_sample_pack": (C.c_int, [P, C.POINTER(rad_sampling), P, P, C.c_int32]),
    "rad_sample_pack_static": (C.c_int, [P, C.POINTER(rad_sampling), P, P]),
    "rad_forward_sample": (C.c_int, [P, C.POINTER(rad_layer), C.POINTER(rad_sampling), P, P, P, P, P]),
    "rad_backward_dW": (C.c_int, [P, C.POINTER(rad_layer), P, P, P, P, C.c_float]),
    "rad_backward_dX": (C.c_int, [P, C.POINTER(rad_layer), P, P, P, P]),
    "rad_softmax_ce": (C.c_int, [P, P, P, C.c_int64, C.c_int64, C.c_int32, P, P]),
    "rad_model_create_mlp": (C.c_int, [P, C.c_int32, C.c_int64, C.c_int32, C.POINTER(C.c_int64), C.c_int32,
                                       C.c_int32, C.c_double, C.POINTER(P)]),
    "rad_model_create_rnn": (C.c_int, [P, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_int32,
                                       C.c_double, C.POINTER(P)]),
    "rad_model_create_cnn": (C.c_int, [P, C.c_int64, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                       C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double,
                                       C.POINTER(P)]),
    "rad_model_destroy": (C.c_int, [P]),
    "rad_model_num_stores": (C.c_int32, [P]),
    "rad_model_store": (P, [P, C.c_int32]),
    "rad_store_set_index_free": (C.c_int, [P, P, C.c_int32]),
    "rad_model_set_index_free": (C.c_int, [P, P, C.c_int32]),
    "rad_model_logits": (P, [P]),
    "rad_model_export_pool_arg": (C.c_int, [P, P, C.c_int32, P]),
    "rad_train_step": (C.c_int, [P, P, C.POINTER(rad_sampling), P, P, C.POINTER(P), C.POINTER(P),
                                 C.POINTER(C.c_float)]),
    "rad_pde_workspace_bytes": (C.c_int, [P, C.POINTER(rad_pde_grid), C.c_double, C.c_int32, C.POINTER(C.c_uint64)]),
    "rad_pde_gradient": (C.c_int, [P, C.POINTER(rad_pde_grid), C.c_int32, P, C.c_double, C.c_uint64, C.c_uint32, P,
                                   C.c_uint64, P, P, P]),
    "rad_path_sample_gradient": (C.c_int, [P, C.POINTER(rad_graph), C.c_int32, P, C.c_int32, C.c_int32, C.c_uint64,
                                           C.c_uint32, P, P]),
    "rad_optimizer_step": (C.c_int, [P, C.POINTER(rad_optimizer), C.c_int64, C.c_int32, C.c_int32,
                                     C.POINTER(C.c_int64), C.POINTER(P), C.POINTER(P), C.POINTER(P), C.POINTER(P),
                                     C.POINTER(P)]),
}

_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("librad_hip.so is missing: run `python -m paper_2007_10412_amd.build` "
                               "(there is no CPU fallback)")
        # torch ships its own HIP runtime under the same soname; it must be in the
        # process first so that this library binds to that one and not to a second copy
        import torch  # noqa: F401
        _lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(_lib, name)
            fn.restype, fn.argtypes = res, args
    return _lib


class RadError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < 7 else status, text))
        self.status = status


def _check(ctx, status):
    if status != RAD_OK:
        raise RadError(status, lib().rad_last_error(ctx).decode() if ctx else "")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def make_layer(batch, d_in, d_out, dtype=RAD_F32, relu=True, has_bias=False, conv=None):
    L = rad_layer(RAD_LINEAR, dtype, batch, d_in, d_out, int(relu), int(has_bias), 0, 0, 0, 0, 0, 0, 0)
    if conv is not None:
        L.kind = RAD_CONV2D
        L.c_in, L.h, L.w, L.c_out, L.kh, L.kw, L.pad = conv
    return L


def make_sampling(scheme, p, seed, stream_id=0, step=0):
    return rad_sampling(scheme, p, seed, stream_id, step)


def rad_fixed_k(p, d):
    return lib().rad_fixed_k(p, d)


def rad_ctx_create(stream=None):
    """stream: a torch.cuda.Stream (its HIP stream is borrowed) or None for the default stream."""
    ctx = P()
    handle = C.c_void_p(stream.cuda_stream) if stream is not None else None
    st = lib().rad_ctx_create(C.byref(ctx), handle)
    if st != RAD_OK:
        raise RadError(st, "rad_ctx_create failed (is a gfx950 device present?)")
    return ctx


def rad_last_error(ctx):
    return lib().rad_last_error(ctx).decode()


def rad_ctx_destroy(ctx):
    _check(None, lib().rad_ctx_destroy(ctx))


def rad_ctx_synchronize(ctx):
    _check(ctx, lib().rad_ctx_synchronize(ctx))


def rad_ctx_timing(ctx, filt):
    _check(ctx, lib().rad_ctx_timing(ctx, None if filt is None else filt.encode()))


def rad_ctx_timing_reset(ctx):
    _check(ctx, lib().rad_ctx_timing_reset(ctx))


def rad_ctx_timing_read(ctx, name):
    n, ms = C.c_int64(), C.c_double()
    _check(ctx, lib().rad_ctx_timing_read(ctx, None if name is None else name.encode(), C.byref(n), C.byref(ms)))
    return n.value, ms.value


def rad_ctx_timing_read_flops(ctx, name):
    a, x = C.c_double(), C.c_double()
    _check(ctx, lib().rad_ctx_timing_read_flops(ctx, None if name is None else name.encode(), C.byref(a), C.byref(x)))
    return a.value, x.value


def rad_probe_ceiling(ctx, kind, operands, sink, nbytes, reps=10):
    out = C.c_double(0.0)
    _check(ctx, lib().rad_probe_ceiling(ctx, kind, _ptr(operands), _ptr(sink), nbytes, reps, C.byref(out)))
    return out.value


def rad_debug_key_shift(ctx, shift):
    _check(ctx, lib().rad_debug_key_shift(ctx, shift))


def rad_store_create(ctx, layer, scheme, p, steps=1):
    s = P()
    _check(ctx, lib().rad_store_create(ctx, C.byref(layer), scheme, p, steps, C.byref(s)))
    return s


def rad_store_destroy(store):
    lib().rad_store_destroy(store)


def rad_store_get_stats(ctx, store):
    st = rad_store_stats()
    _check(ctx, lib().rad_store_get_stats(ctx, store, C.byref(st)))
    return {k: getattr(st, k) for k, _ in rad_store_stats._fields_}


def rad_store_export_csr(ctx, store, rows):
    """Returns (row_ptr int64 [rows+1], col int32 [nnz], val float32 [nnz]) as numpy arrays."""
    nnz = rad_store_get_stats(ctx, store)["nnz"]
    row_ptr = np.zeros(rows + 1, dtype=np.int64)
    col = np.zeros(max(nnz, 1), dtype=np.int32)
    val = np.zeros(max(nnz, 1), dtype=np.float32)
    _check(ctx, lib().rad_store_export_csr(ctx, store, row_ptr.ctypes.data, col.ctypes.data, val.ctypes.data, nnz))
    return row_ptr, col[:nnz], val[:nnz]


def rad_store_export_bits(ctx, store, rows, d_out):
    words = np.zeros((rows, (d_out + 31) // 32), dtype=np.uint32)
    _check(ctx, lib().rad_store_export_bits(ctx, store, words.ctypes.data))
    return words


def rad_store_import_bits(ctx, store, words):
    words = np.ascontiguousarray(words, dtype=np.uint32)
    _check(ctx, lib().rad_store_import_bits(ctx, store, words.ctypes.data))


def rad_sample_pack(ctx, sampling, x, store, step_slot=0):
    _check(ctx, lib().rad_sample_pack(ctx, C.byref(sampling), _ptr(x), store, step_slot))


def rad_sample_pack_static(ctx, sampling, x, store):
    _check(ctx, lib().rad_sample_pack_static(ctx, C.byref(sampling), _ptr(x), store))


def rad_forward_sample(ctx, layer, sampling, x, W, bias, y, store):
    _check(ctx, lib().rad_forward_sample(ctx, C.byref(layer), C.byref(sampling), _ptr(x), _ptr(W), _ptr(bias),
                                         _ptr(y), store))


def rad_backward_dW(ctx, layer, store, dy, dW, dbias=None, beta=0.0):
    _check(ctx, lib().rad_backward_dW(ctx, C.byref(layer), store, _ptr(dy), _ptr(dW), _ptr(dbias), beta))


def rad_backward_dX(ctx, layer, store, dy, W, dX):
    _check(ctx, lib().rad_backward_dX(ctx, C.byref(layer), store, _ptr(dy), _ptr(W), _ptr(dX)))


def rad_softmax_ce(ctx, logits, labels, dtype, dlogits, loss_dev):
    rows, classes = logits.shape
    _check(ctx, lib().rad_softmax_ce(ctx, _ptr(logits), _ptr(labels), rows, classes, dtype, _ptr(dlogits),
                                     _ptr(loss_dev)))


def rad_model_create_mlp(ctx, dtype, batch, dims, has_bias, scheme, p):
    m = P()
    arr = (C.c_int64 * len(dims))(*dims)
    _check(ctx, lib().rad_model_create_mlp(ctx, dtype, batch, len(dims) - 1, arr, int(has_bias), scheme, p,
                                           C.byref(m)))
    return m


def rad_model_create_rnn(ctx, batch, T, d_input, hidden, classes, scheme, p):
    m = P()
    _check(ctx, lib().rad_model_create_rnn(ctx, batch, T, d_input, hidden, classes, scheme, p, C.byref(m)))
    return m


def rad_model_create_cnn(ctx, batch, channels, pool, ksize, height, width, classes, scheme, p):
    m = P()
    n_conv = len(channels) - 1
    ch = (C.c_int32 * len(channels))(*channels)
    pl = (C.c_int32 * n_conv)(*[int(v) for v in pool])
    _check(ctx, lib().rad_model_create_cnn(ctx, batch, n_conv, ch, pl, ksize, height, width, classes, scheme, p,
                                           C.byref(m)))
    return m


def rad_model_destroy(model):
    lib().rad_model_destroy(model)


def rad_model_num_stores(model):
    return lib().rad_model_num_stores(model)


def rad_model_store(model, l):
    return C.c_void_p(lib().rad_model_store(model, l))


def rad_model_export_pool_arg(ctx, model, l, n):
    out = np.zeros(n, dtype=np.uint8)
    _check(ctx, lib().rad_model_export_pool_arg(ctx, model, l, out.ctypes.data))
    return out


def rad_store_set_index_free(ctx, store, on=True):
    _check(ctx, lib().rad_store_set_index_free(ctx, store, 1 if on else 0))


def rad_model_set_index_free(ctx, model, on=True):
    _check(ctx, lib().rad_model_set_index_free(ctx, model, 1 if on else 0))


def rad_model_logits(model):
    return lib().rad_model_logits(model)


def rad_train_step(ctx, model, sampling, x, labels, params, grads, want_loss=True):
    """params/grads: lists of torch tensors in the model's documented order.  Returns the loss (float), or
    None with want_loss=False: the step is then only enqueued (loss_host = null)."""
    n = len(params)
    pa = (P * n)(*[p.data_ptr() for p in params])
    ga = (P * n)(*[g.data_ptr() for g in grads])
    if not want_loss:
        _check(ctx, lib().rad_train_step(ctx, model, C.byref(sampling), _ptr(x), _ptr(labels), pa, ga, None))
        return None
    loss = C.c_float()
    _check(ctx, lib().rad_train_step(ctx, model, C.byref(sampling), _ptr(x), _ptr(labels), pa, ga, C.byref(loss)))
    return loss.value


def make_optimizer(kind, lr, l2=0.0, beta1=0.9, beta2=0.999, eps=1e-8):
    return rad_optimizer(kind, lr, l2, beta1, beta2, eps)


def rad_optimizer_step(ctx, opt, t, dtype, params, grads, m=None, v=None, master=None):
    """params, grads, m, v, master: lists of torch tensors (m, v for RAD_ADAM; master for RAD_BF16)."""
    n = len(params)

    def arr(ts):
        return None if ts is None else (P * n)(*[x.data_ptr() for x in ts])
    counts = (C.c_int64 * n)(*[int(x.numel()) for x in params])
    _check(ctx, lib().rad_optimizer_step(ctx, C.byref(opt), int(t), dtype, n, counts, arr(params), arr(grads), arr(m),
                                         arr(v), arr(master)))


def make_pde_grid(n=32, steps=40960, D=0.25, dt=1.0 / 4096):
    return rad_pde_grid(n, steps, D, dt)


def rad_pde_workspace_bytes(ctx, grid, p, problems):
    out = C.c_uint64()
    _check(ctx, lib().rad_pde_workspace_bytes(ctx, C.byref(grid), p, problems, C.byref(out)))
    return out.value


def rad_pde_gradient(ctx, grid, theta, p, seed, stream_id, workspace, loss, grad, stored=None):
    """theta [problems, 7] fp64 device tensor; workspace a device byte tensor; loss [problems], grad [problems, 7]
    fp64, stored [problems] int64 or None."""
    problems = int(theta.shape[0])
    _check(ctx, lib().rad_pde_gradient(ctx, C.byref(grid), problems, _ptr(theta), p, seed, stream_id, _ptr(workspace),
                                       int(workspace.numel() * workspace.element_size()), _ptr(loss), _ptr(grad),
                                       _ptr(stored)))


def rad_path_sample_gradient(ctx, level_ptr, succ_ptr, succ, partial, y, inputs, k, seed, stream_id, adjoint, reached):
    """level_ptr: host sequence of ints; succ_ptr, succ (int32), partial (fp64), inputs (int32): device tensors;
    adjoint (fp64) and reached (int32 storage) device tensors of n_vertices entries."""
    lp = (C.c_int32 * len(level_ptr))(*[int(v) for v in level_ptr])
    g = rad_graph(int(succ_ptr.numel()) - 1, len(level_ptr) - 1, int(succ.numel()), C.cast(lp, P), succ_ptr.data_ptr(),
                  succ.data_ptr(), partial.data_ptr())
    _check(ctx, lib().rad_path_sample_gradient(ctx, C.byref(g), int(y), _ptr(inputs), int(inputs.numel()), int(k), seed,
                                               stream_id, _ptr(adjoint), _ptr(reached)))
