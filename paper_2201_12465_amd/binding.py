"""ctypes binding of libflmi355.so (the product: include/fl_layer.h) and of
libflmi355_test.so (the same code plus the test-only entry points of
include/fl_test.h): same names as the headers, argument marshalling only.  Every
computation runs in the library's HIP kernels; there is no fallback: if a library
is missing, loading raises.

lib() is the product library and what Layer, opt_step, ... use by default;
test_lib() is the test build.  Each library is a process of its own as far as
state goes (allocator, side streams, last error): a handle created through one
must be used through the same one, which is why every helper takes the library
as an optional last argument.

Device buffers are passed as integers (addresses) or as objects with a
``data_ptr()`` method (torch tensors); streams as integers (``hipStream_t``).
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflmi355.so")
TEST_LIB_PATH = os.path.join(_HERE, "libflmi355_test.so")

FL_OK, FL_ERR_INVALID_ARG, FL_ERR_UNSUPPORTED, FL_ERR_OOM, FL_ERR_DEVICE, FL_ERR_STATE = range(6)
FL_F32, FL_BF16 = 0, 1
FL_ACT_RELU, FL_ACT_GELU = 0, 1
FL_NORM_POST, FL_NORM_PRE = 0, 1
PARAM_FIELDS = ("Wqkv", "bqkv", "Wo", "bo", "W1", "b1", "W2", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")
KERNEL_CLASSES = ("gemm_nt", "gemm_nn", "gemm_tn", "splitk_reduce", "attn_fwd", "attn_bwd",
                  "ln_fwd", "ln_bwd", "colsum", "wt_transpose")


class FlError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"fl status {status}: {message}")
        self.status = status


class fl_layer_config_t(C.Structure):
    _fields_ = [("max_B", C.c_int32), ("max_T", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ffn", C.c_int32), ("act", C.c_int), ("norm", C.c_int), ("dtype", C.c_int),
                ("ln_eps", C.c_float), ("causal", C.c_int32)]


class fl_layer_params_t(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_FIELDS]


class fl_layer_grads_t(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_FIELDS]


class fl_alloc_stats_t(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("backing_mallocs", "backing_bytes", "cache_hits", "cache_misses",
                                           "live_bytes", "peak_bytes", "cached_bytes", "split_count",
                                           "requested_bytes", "largest_free_block", "free_blocks")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class fl_alloc_event_t(C.Structure):
    _fields_ = [("seq", C.c_uint64), ("ptr", C.c_uint64), ("requested", C.c_uint64), ("granted", C.c_uint64),
                ("tag", C.c_int32), ("kind", C.c_int32)]


OP_KINDS = ("none", "linear_fwd", "attention_fwd", "layernorm_fwd", "linear_bwd", "attention_bwd", "layernorm_bwd")
ALLOC_EVENT_KINDS = ("from_cache", "from_device", "release")


class fl_opt_config_t(C.Structure):
    _fields_ = [("kind", C.c_int), ("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("step", C.c_int32)]


class fl_prof_entry_t(C.Structure):
    _fields_ = [("kernel_class", C.c_int32), ("launches", C.c_int32), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double), ("empty_bracket_ms", C.c_double)]


BACKING_MALLOC = C.CFUNCTYPE(C.c_int, C.POINTER(C.c_void_p), C.c_size_t)
BACKING_FREE = C.CFUNCTYPE(C.c_int, C.c_void_p)

_lib = None
_test_lib = None


def _signatures():
    vp, i32, i64, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float
    product = {
        "fl_layer_create": (C.c_int, [C.POINTER(fl_layer_config_t), C.POINTER(vp)]),
        "fl_layer_forward": (C.c_int, [vp, C.POINTER(fl_layer_params_t), vp, vp, i32, i32, vp, vp]),
        "fl_layer_forward_static": (C.c_int, [vp, C.POINTER(fl_layer_params_t), vp, vp, i32, i32, vp, vp]),
        "fl_layer_backward": (C.c_int, [vp, C.POINTER(fl_layer_params_t), vp, vp, C.POINTER(fl_layer_grads_t), vp]),
        "fl_layer_backward_accumulate": (C.c_int, [vp, C.POINTER(fl_layer_params_t), vp, vp,
                                                   C.POINTER(fl_layer_grads_t), i32, vp]),
        "fl_opt_step": (C.c_int, [C.POINTER(fl_opt_config_t), C.c_int, i32, C.POINTER(vp), C.POINTER(vp),
                                  C.POINTER(vp), C.POINTER(vp), C.POINTER(i64), vp]),
        "fl_opt_step_master": (C.c_int, [C.POINTER(fl_opt_config_t), C.c_int, i32, C.POINTER(vp), C.POINTER(vp),
                                         C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(i64), vp]),
        "fl_zero_grad": (C.c_int, [C.c_int, i32, C.POINTER(vp), C.POINTER(i64), vp]),
        "fl_layer_set_dropout": (C.c_int, [vp, f32, f32, u64]),
        "fl_layer_destroy": (C.c_int, [vp]),
        "fl_last_error": (C.c_char_p, []),
        "fl_alloc_get_stats": (C.c_int, [C.POINTER(fl_alloc_stats_t)]),
        "fl_alloc_trace_enable": (C.c_int, [i32]),
        "fl_alloc_trace_read": (C.c_int, [C.POINTER(fl_alloc_event_t), i32, C.POINTER(i32)]),
        "fl_set_grad_overlap": (C.c_int, [i32]),
        "fl_alloc_trim": (C.c_int, []),
        "fl_layer_set_deferred_join": (C.c_int, [vp, i32]),
        "fl_layer_join": (C.c_int, [vp, vp]),
        "fl_alloc_set_split_limit": (C.c_int, [u64]),
        "fl_prof_enable": (C.c_int, [C.c_uint32]),
        "fl_prof_collect": (C.c_int, [C.POINTER(fl_prof_entry_t), i32, C.POINTER(i32)]),
    }
    test = {
        "fl_test_gemm": (i32, [i32, i32, i32, vp, vp, vp, i32, i32, i32, vp, vp, i32, vp, i32, vp, i32, vp, vp]),
        "fl_test_gemm_time": (i32, [i32, i32, i32, vp, vp, vp, i32, i32, i32, i32, vp, i32, C.POINTER(f32), vp]),
        "fl_test_gemm_force_variant": (None, [i32]),
        "fl_test_gemm_force_tile_height": (None, [i32]),
        "fl_test_gemm_splits": (i32, [i32, i32, i32, i32]),
        "fl_test_layernorm_fwd": (i32, [i32, vp, vp, vp, f32, i32, i32, vp, vp, vp, vp]),
        "fl_test_layernorm_bwd_ws_floats": (i32, [i32, i32]),
        "fl_test_layernorm_bwd": (i32, [i32, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp]),
        "fl_test_copy": (i32, [vp, vp, u64, vp]),
        "fl_test_mfma_probe": (i32, [i32, i32, i32, vp, C.POINTER(C.c_double), vp]),
        "fl_test_gemm_variant": (i32, [i32, i32, i32, i32, i32]),
        "fl_test_gemm_variant_forward": (i32, [i32, i32, i32]),
        "fl_test_gemm_f32_small": (i32, [i32, i32]),
        "fl_test_attention_path": (i32, [i32, i32]),
        "fl_test_transpose_bf16": (i32, [i32, vp, vp, vp, vp, vp]),
        "fl_test_colsum_ws_floats": (i64, [i32, i32]),
        "fl_test_colsum": (i32, [i32, vp, i32, i32, vp, vp, vp]),
        "fl_test_attention_fwd": (i32, [i32, vp, vp, i32, f32, u64, i32, i32, i32, i32, vp, vp, vp]),
        "fl_test_attention_bwd": (i32, [i32, vp, vp, vp, vp, vp, i32, f32, u64, i32, i32, i32, i32, vp, vp, vp]),
        "fl_test_dropout_mul": (i32, [i32, vp, vp, i32, i32, i32, f32, u64, vp]),
        "fl_test_attention_force_general": (None, [i32]),
        "fl_test_attention_force_unfused_bwd": (None, [i32]),
        "fl_test_layer_peek_linear": (i32, [vp, i32, vp, u64, C.POINTER(u64), vp]),
        "fl_test_alloc_create": (vp, [BACKING_MALLOC, BACKING_FREE]),
        "fl_test_alloc_destroy": (None, [vp]),
        "fl_test_alloc_alloc": (vp, [vp, u64, vp]),
        "fl_test_alloc_release": (i32, [vp, vp]),
        "fl_test_alloc_trim": (None, [vp]),
        "fl_test_alloc_set_split_limit": (None, [vp, u64]),
        "fl_test_alloc_stats": (None, [vp, C.POINTER(fl_alloc_stats_t)]),
        "fl_test_alloc_alloc_tagged": (vp, [vp, u64, vp, i32]),
        "fl_test_alloc_trace_enable": (None, [vp, i32]),
        "fl_test_alloc_trace_read": (i32, [vp, C.POINTER(fl_alloc_event_t), i32]),
        "fl_test_tape_replay": (i32, [i32, C.POINTER(i32), C.POINTER(i32), i32, i32, C.POINTER(i32),
                                      C.POINTER(i32), C.POINTER(i32), i32]),
    }
    return product, test


def _load(path: str, with_test: bool) -> C.CDLL:
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python -m paper_2201_12465_amd.build`")
    L = C.CDLL(path)
    product, test = _signatures()
    sig = dict(product, **test) if with_test else product
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    return L


def lib() -> C.CDLL:
    """Loads the product library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        _lib = _load(LIB_PATH, False)
    return _lib


def test_lib() -> C.CDLL:
    """Loads the test build of the library (once): the product's entry points plus include/fl_test.h."""
    global _test_lib
    if _test_lib is None:
        _test_lib = _load(TEST_LIB_PATH, True)
    return _test_lib


def ptr(x) -> int | None:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def check(status: int, L=None) -> None:
    if status != FL_OK:
        raise FlError(status, (L or lib()).fl_last_error().decode())


def _pack(struct_type, tensors: dict):
    s = struct_type()
    for n in PARAM_FIELDS:
        setattr(s, n, ptr(tensors[n]))
    return s


class Layer:
    """Thin handle wrapper: create / forward / backward / destroy."""

    def __init__(self, max_B, max_T, d_model, n_heads, d_ffn, act="relu", norm="post", dtype="f32", ln_eps=1e-5,
                 causal=False, L=None):
        self._L = L or lib()
        cfg = fl_layer_config_t(max_B, max_T, d_model, n_heads, d_ffn,
                                {"relu": FL_ACT_RELU, "gelu": FL_ACT_GELU}[act],
                                {"post": FL_NORM_POST, "pre": FL_NORM_PRE}[norm],
                                {"f32": FL_F32, "bf16": FL_BF16}[dtype], ln_eps, 1 if causal else 0)
        self._h = C.c_void_p()
        check(self._L.fl_layer_create(C.byref(cfg), C.byref(self._h)), self._L)

    def set_dropout(self, p_attn: float, p_hidden: float, seed: int) -> None:
        check(self._L.fl_layer_set_dropout(self._h, p_attn, p_hidden, seed), self._L)

    def forward(self, params: dict, X, lengths, B: int, T: int, Y, stream: int = 0) -> None:
        p = _pack(fl_layer_params_t, params)
        check(self._L.fl_layer_forward(self._h, C.byref(p), ptr(X), ptr(lengths), B, T, ptr(Y), stream), self._L)

    def forward_static(self, params: dict, X, lengths, B: int, T: int, Y, stream: int = 0) -> None:
        p = _pack(fl_layer_params_t, params)
        check(self._L.fl_layer_forward_static(self._h, C.byref(p), ptr(X), ptr(lengths), B, T, ptr(Y), stream), self._L)

    def backward(self, params: dict, dY, dX, grads: dict, stream: int = 0, accumulate: bool = False) -> None:
        p = _pack(fl_layer_params_t, params)
        g = _pack(fl_layer_grads_t, grads)
        if accumulate:
            check(self._L.fl_layer_backward_accumulate(self._h, C.byref(p), ptr(dY), ptr(dX), C.byref(g), 1, stream), self._L)
        else:
            check(self._L.fl_layer_backward(self._h, C.byref(p), ptr(dY), ptr(dX), C.byref(g), stream), self._L)

    def set_deferred_join(self, enabled: bool) -> None:
        check(self._L.fl_layer_set_deferred_join(self._h, 1 if enabled else 0), self._L)

    def join(self, stream: int = 0) -> None:
        check(self._L.fl_layer_join(self._h, stream), self._L)

    def peek_linear(self, lin: int, dst, stream: int = 0) -> int:
        """Test build only: copies the recorded forward's lin-th linear output into dst; returns its byte size."""
        n = C.c_uint64(0)
        cap = dst.numel() * dst.element_size()
        check(self._L.fl_test_layer_peek_linear(self._h, lin, ptr(dst), cap, C.byref(n), stream), self._L)
        return int(n.value)

    def destroy(self) -> None:
        if self._h:
            check(self._L.fl_layer_destroy(self._h), self._L)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


FL_OPT_SGD, FL_OPT_ADAM = 0, 1


def _ptr_array(items):
    if items is None:
        return None
    return (C.c_void_p * len(items))(*[ptr(x) for x in items])


def opt_step(kind: str, dtype: str, params, grads, state_m, state_v, numel, stream: int = 0, *, lr, momentum=0.0,
             weight_decay=0.0, beta1=0.9, beta2=0.999, eps=1e-8, step=1, master=None) -> None:
    """One fused optimizer step over lists of tensors (see fl_opt_step; with `master`, fl_opt_step_master)."""
    cfg = fl_opt_config_t({"sgd": FL_OPT_SGD, "adam": FL_OPT_ADAM}[kind], lr, momentum, weight_decay, beta1, beta2,
                          eps, step)
    n = len(params)
    ne = (C.c_int64 * n)(*[int(x) for x in numel])
    if master is not None:
        check(lib().fl_opt_step_master(C.byref(cfg), {"f32": FL_F32, "bf16": FL_BF16}[dtype], n, _ptr_array(params),
                                       _ptr_array(master), _ptr_array(grads), _ptr_array(state_m),
                                       _ptr_array(state_v), ne, stream))
        return
    check(lib().fl_opt_step(C.byref(cfg), {"f32": FL_F32, "bf16": FL_BF16}[dtype], n, _ptr_array(params),
                            _ptr_array(grads), _ptr_array(state_m), _ptr_array(state_v), ne, stream))


def zero_grad(dtype: str, grads, numel, stream: int = 0) -> None:
    n = len(grads)
    ne = (C.c_int64 * n)(*[int(x) for x in numel])
    check(lib().fl_zero_grad({"f32": FL_F32, "bf16": FL_BF16}[dtype], n, _ptr_array(grads), ne, stream))


def alloc_stats(L=None) -> dict:
    s = fl_alloc_stats_t()
    check((L or lib()).fl_alloc_get_stats(C.byref(s)), L)
    return s.as_dict()


def events_as_dicts(ev, n) -> list:
    return [{"seq": int(e.seq), "ptr": int(e.ptr), "requested": int(e.requested), "granted": int(e.granted),
             "op": OP_KINDS[e.tag & 0xFF], "node": e.tag >> 8, "kind": ALLOC_EVENT_KINDS[e.kind]} for e in ev[:n]]


def alloc_trace_enable(capacity: int, L=None) -> None:
    check((L or lib()).fl_alloc_trace_enable(capacity), L)


def alloc_trace_read(cap: int = 4096, L=None) -> list:
    ev = (fl_alloc_event_t * cap)()
    n = C.c_int32(0)
    check((L or lib()).fl_alloc_trace_read(ev, cap, C.byref(n)), L)
    return events_as_dicts(ev, n.value)


def set_grad_overlap(enabled: bool, L=None) -> None:
    check((L or lib()).fl_set_grad_overlap(1 if enabled else 0), L)


def alloc_trim(L=None) -> None:
    check((L or lib()).fl_alloc_trim(), L)


def alloc_set_split_limit(nbytes: int, L=None) -> None:
    check((L or lib()).fl_alloc_set_split_limit(nbytes), L)


def prof_enable(classes=None, L=None) -> None:
    """classes: iterable of names from KERNEL_CLASSES, "all", or None/empty to disable."""
    mask = 0
    if classes == "all":
        mask = (1 << len(KERNEL_CLASSES)) - 1
    elif classes:
        for c in classes:
            mask |= 1 << KERNEL_CLASSES.index(c)
    check((L or lib()).fl_prof_enable(mask), L)


def prof_collect(L=None) -> dict:
    arr = (fl_prof_entry_t * len(KERNEL_CLASSES))()
    n = C.c_int32(0)
    check((L or lib()).fl_prof_collect(arr, len(KERNEL_CLASSES), C.byref(n)), L)
    return {KERNEL_CLASSES[arr[i].kernel_class]: {"launches": arr[i].launches, "total_ms": arr[i].total_ms,
                                                  "flops": arr[i].flops, "bytes": arr[i].bytes,
                                                  "empty_bracket_ms": arr[i].empty_bracket_ms}
            for i in range(n.value)}
