"""ctypes binding of libms.so: same names as include/ms.h, argument marshalling only.

Every step of the hot path (space description, sampling, interpretation,
validation, kernel materialisation, launch, measurement, search) runs inside
the library; this module only converts Python values to the C structs.
There is no CPU fallback: if the library is missing, loading raises.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libms.so")

MS_OK, MS_ERR_BAD_ARG, MS_ERR_INVALID_TRACE, MS_ERR_UNSUPPORTED, MS_ERR_COMPILE, MS_ERR_HIP, MS_ERR_NOMEM = range(7)
(OP_GEMM, OP_BMM_NT, OP_BMM_NN, OP_CONV2D_NHWC, OP_DWCONV2D_NHWC, OP_SOFTMAX, OP_NORM,
 OP_CONV2D_TRANSPOSED_NHWC, OP_CONV1D_NWC, OP_CONV3D_NDHWC) = range(10)
F32, F16, BF16, I8, I32 = range(5)
SLOT_PERFECT_TILE, SLOT_CATEGORICAL = 0, 1
(SLOT_TENSORIZE, SLOT_TILE_I, SLOT_TILE_J, SLOT_TILE_C, SLOT_TILE_K, SLOT_UNROLL, SLOT_CACHE_READ, SLOT_VECTORIZE,
 SLOT_STORAGE_ALIGN, SLOT_REORDER, SLOT_VECTORIZE_B, SLOT_CACHE_WRITE, SLOT_COMPUTE_AT, SLOT_RFACTOR) = range(14)
SPACE_TENSORIZE, SPACE_CACHE_READ, SPACE_VECTORIZE, SPACE_UNROLL, SPACE_STORAGE_ALIGN, SPACE_REORDER, SPACE_CACHE_WRITE = 1, 2, 4, 8, 16, 32, 64
SPACE_COMPUTE_AT = 128
SPACE_TENSORIZE_F32 = 0x100  # opt-in: fp32 operators on the fp32 matrix-core intrinsics
SPACE_TAP_ROWS = 0x200  # opt-in: conv2d reduction laid out as filter rows (first layers with few input channels)
SPACE_RFACTOR = 0x400  # opt-in: sample the split of the reduction across workgroups (needs a workspace)
SPACE_DEFAULT = 0xFF
STATIC_WORKSPACE_BYTES = 32 << 20
FAM_GEMM_ALU, FAM_GEMM_MFMA, FAM_DWCONV, FAM_REDUCE = range(4)
MAX_SLOTS, MAX_FACTORS, MAX_CANDS, MAX_LOOPS = 16, 4, 12, 8

F8E4M3 = 5
DTYPE_NAMES = {"f32": F32, "f16": F16, "bf16": BF16, "i8": I8, "i32": I32, "f8": F8E4M3}


class MsError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("ms error %d: %s" % (code, msg))
        self.code = code


class ms_op_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("in_dtype", C.c_int32), ("out_dtype", C.c_int32), ("stride", C.c_int32),
                ("pad", C.c_int32), ("has_bias", C.c_int32), ("relu", C.c_int32), ("dilation", C.c_int32),
                ("dims", C.c_int64 * 8), ("a_strides", C.c_int64 * 3), ("b_strides", C.c_int64 * 3)]


class ms_loop(C.Structure):
    _fields_ = [("name", C.c_char * 8), ("extent", C.c_int64), ("is_reduction", C.c_int32), ("reserved", C.c_int32)]


class ms_slot(C.Structure):
    _fields_ = [("slot_id", C.c_int32), ("kind", C.c_int32), ("name", C.c_char * 16), ("extent", C.c_int64),
                ("n_factors", C.c_int32), ("n_candidates", C.c_int32), ("candidates", C.c_int64 * MAX_CANDS),
                ("weight", C.c_int32 * MAX_CANDS), ("depends_on", C.c_int32), ("reserved", C.c_int32),
                ("extent_by_choice", C.c_int64 * MAX_CANDS)]


class ms_module_info(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("primitives", C.c_char * 96), ("location", C.c_int32), ("flag", C.c_uint32),
                ("requires", C.c_uint32), ("reserved", C.c_int32)]


class ms_space(C.Structure):
    _fields_ = [("family", C.c_int32), ("flags", C.c_uint32), ("n_slots", C.c_int32), ("reserved", C.c_int32),
                ("slots", ms_slot * MAX_SLOTS)]


class ms_decision(C.Structure):
    _fields_ = [("slot_id", C.c_int32), ("kind", C.c_int32), ("n", C.c_int32), ("reserved", C.c_int32),
                ("v", C.c_int64 * MAX_FACTORS)]


class ms_trace(C.Structure):
    _fields_ = [("n", C.c_int32), ("reserved", C.c_int32), ("d", ms_decision * MAX_SLOTS)]

    def copy(self):
        t = ms_trace()
        C.memmove(C.byref(t), C.byref(self), C.sizeof(ms_trace))
        return t

    def decisions(self):
        return [(self.d[i].slot_id, [int(self.d[i].v[k]) for k in range(self.d[i].n)]) for i in range(self.n)]


class ms_variant_params(C.Structure):
    _fields_ = [("family", C.c_int32), ("mfma", C.c_int32), ("ti", C.c_int32 * 4), ("tj", C.c_int32 * 4),
                ("tc", C.c_int32 * 4), ("tk", C.c_int32 * 4), ("tile_unit", C.c_int32 * 3), ("block_m", C.c_int32),
                ("block_n", C.c_int32), ("block_k", C.c_int32), ("grid", C.c_int32 * 3), ("threads", C.c_int32),
                ("waves", C.c_int32), ("acc_per_thread", C.c_int32), ("lds_bytes", C.c_int32),
                ("cache_read", C.c_int32), ("vec", C.c_int32), ("unroll", C.c_int32), ("unroll_k1", C.c_int32),
                ("unroll_k2", C.c_int32), ("lds_pad", C.c_int32), ("reorder", C.c_int32), ("vec_b", C.c_int32), ("cache_write", C.c_int32), ("compute_at", C.c_int32), ("tap_rows", C.c_int32), ("rfactor", C.c_int32), ("reserved", C.c_int32 * 3),
                ("key", C.c_uint64)]

    def as_dict(self):
        out = {}
        for name, _ in self._fields_:
            v = getattr(self, name)
            out[name] = list(v) if hasattr(v, "__len__") else v
        return out


class ms_variant_resources(C.Structure):
    _fields_ = [("vgprs", C.c_int32), ("agprs", C.c_int32), ("sgprs", C.c_int32), ("scratch_bytes", C.c_int32),
                ("spilled_vgprs", C.c_int32), ("lds_bytes", C.c_int32), ("reserved", C.c_int32 * 2)]


class ms_limits(C.Structure):
    _fields_ = [("max_threads", C.c_int32), ("max_lds_bytes", C.c_int32), ("max_acc_per_thread", C.c_int32),
                ("wave_size", C.c_int32), ("max_waves", C.c_int32), ("reserved", C.c_int32 * 3)]


class ms_bufset(C.Structure):
    _fields_ = [("inputs", C.c_void_p * 4), ("output", C.c_void_p), ("workspace", C.c_void_p)]


class ms_measure_cfg(C.Structure):
    _fields_ = [("warmup", C.c_int32), ("repeats", C.c_int32), ("launches_per_repeat", C.c_int32),
                ("instances", C.c_int32)]


class ms_measure_result(C.Structure):
    _fields_ = [("min_us", C.c_double), ("median_us", C.c_double), ("mean_us", C.c_double), ("flop", C.c_double),
                ("bytes", C.c_double), ("n", C.c_int32), ("reserved", C.c_int32)]


class ms_search_cfg(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("trials", C.c_int32), ("init_population", C.c_int32), ("population", C.c_int32),
                ("children", C.c_int32), ("eps_permille", C.c_int32), ("compile_threads", C.c_int32),
                ("temperature0", C.c_double), ("temperature1", C.c_double), ("measure", ms_measure_cfg),
                ("cost_model", C.c_int32), ("model_candidates", C.c_int32), ("model_min_trials", C.c_int32), ("pretrain_n", C.c_int32),
                ("pretrain_X", C.POINTER(C.c_double)), ("pretrain_y", C.POINTER(C.c_double)), ("pretrain_d", C.c_int32),
                ("reserved", C.c_int32)]


class ms_trial(C.Structure):
    _fields_ = [("index", C.c_int32), ("status", C.c_int32), ("us", C.c_double), ("best_us", C.c_double),
                ("trace", ms_trace), ("key", C.c_uint64)]


class ms_search_result(C.Structure):
    _fields_ = [("best_trace", ms_trace), ("best_us", C.c_double), ("best_trial", C.c_int32), ("n_measured", C.c_int32),
                ("n_invalid", C.c_int32), ("n_failed", C.c_int32), ("n_duplicate", C.c_int32), ("reserved", C.c_int32),
                ("wall_seconds", C.c_double)]


class ms_device_info(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("arch", C.c_char * 32), ("compute_units", C.c_int32), ("wave_size", C.c_int32),
                ("lds_bytes_per_block", C.c_int32), ("max_threads_per_block", C.c_int32), ("clock_khz", C.c_int32),
                ("mem_clock_khz", C.c_int32), ("mem_bus_bits", C.c_int32), ("l2_bytes", C.c_int32),
                ("global_mem_bytes", C.c_int64)]


TRIAL_CB = C.CFUNCTYPE(C.c_int32, C.POINTER(ms_trial), C.c_void_p)
LATENCY_FN = C.CFUNCTYPE(C.c_double, C.POINTER(ms_variant_params), C.c_void_p)

# every symbol include/ms.h declares: name -> (restype, argtypes)
_P = C.POINTER
SYMBOLS = {
    "ms_op_create": (C.c_int32, [_P(ms_op_desc), _P(C.c_void_p)]),
    "ms_op_destroy": (None, [C.c_void_p]),
    "ms_op_get_desc": (C.c_int32, [C.c_void_p, _P(ms_op_desc)]),
    "ms_op_loops": (C.c_int32, [C.c_void_p, _P(ms_loop), _P(C.c_int32)]),
    "ms_op_work": (C.c_int32, [C.c_void_p, _P(C.c_double), _P(C.c_double)]),
    "ms_op_tensor_bytes": (C.c_int32, [C.c_void_p, C.c_int32, _P(C.c_int64)]),
    "ms_module_count": (C.c_int32, []),
    "ms_module_get": (C.c_int32, [C.c_int32, _P(ms_module_info)]),
    "ms_space_compose": (C.c_int32, [C.c_void_p, _P(C.c_int32), C.c_int32, _P(C.c_uint32), _P(ms_space)]),
    "ms_space_stochastic_compose": (C.c_int32, [C.c_void_p, _P(C.c_int32), C.c_int32, C.c_uint64, _P(C.c_int32), _P(C.c_int32), _P(ms_space)]),
    "ms_space_describe": (C.c_int32, [C.c_void_p, C.c_uint32, _P(ms_space)]),
    "ms_space_log10_size": (C.c_int32, [_P(ms_space), _P(C.c_double)]),
    "ms_trace_sample": (C.c_int32, [_P(ms_space), C.c_uint64, C.c_uint64, _P(ms_trace)]),
    "ms_trace_sample_valid": (C.c_int32, [C.c_void_p, _P(ms_space), C.c_uint64, C.c_uint64, C.c_int32, _P(ms_trace)]),
    "ms_trace_mutate": (C.c_int32, [_P(ms_space), _P(ms_trace), C.c_uint64, _P(ms_trace)]),
    "ms_trace_to_text": (C.c_int32, [C.c_void_p, _P(ms_space), _P(ms_trace), C.c_char_p, C.c_size_t, _P(C.c_size_t)]),
    "ms_trace_from_text": (C.c_int32, [_P(ms_space), C.c_char_p, _P(ms_trace)]),
    "ms_trace_validate": (C.c_int32, [C.c_void_p, _P(ms_space), _P(ms_trace), _P(ms_variant_params)]),
    "ms_get_limits": (C.c_int32, [_P(ms_limits)]),
    "ms_set_limits": (C.c_int32, [_P(ms_limits)]),
    "ms_variant_build": (C.c_int32, [C.c_void_p, _P(ms_space), _P(ms_trace), _P(C.c_void_p)]),
    "ms_variant_destroy": (None, [C.c_void_p]),
    "ms_variant_info": (C.c_int32, [C.c_void_p, _P(ms_variant_params), _P(C.c_size_t)]),
    "ms_variant_kernel_text": (C.c_int32, [C.c_void_p, _P(ms_variant_params), C.c_char_p, C.c_size_t, _P(C.c_size_t)]),
    "ms_variant_resources_get": (C.c_int32, [C.c_void_p, _P(ms_variant_resources)]),
    "ms_prebuild": (C.c_int32, [C.c_void_p, _P(ms_space), _P(ms_trace), C.c_int32, C.c_int32, _P(C.c_int32)]),
    "ms_set_cache_dir": (C.c_int32, [C.c_char_p]),
    "ms_jit_stats": (C.c_int32, [_P(C.c_int64), _P(C.c_int64), _P(C.c_int64), _P(C.c_int32), _P(C.c_int32)]),
    "ms_variant_launch": (C.c_int32, [C.c_void_p, _P(C.c_void_p), _P(C.c_void_p), C.c_void_p, C.c_int32, C.c_void_p]),
    "ms_variant_prepare": (C.c_int32, [C.c_void_p]),
    "ms_variant_launch_static": (C.c_int32, [C.c_void_p, _P(C.c_void_p), _P(C.c_void_p), C.c_int32, C.c_void_p]),
    "ms_variant_coverage": (C.c_int32, [C.c_void_p, _P(ms_variant_params), C.c_void_p, C.c_int64]),
    "ms_variant_reduction_coverage": (C.c_int32, [C.c_void_p, _P(ms_variant_params), C.c_void_p, C.c_int64, _P(C.c_int64)]),
    "ms_measure": (C.c_int32, [C.c_void_p, _P(ms_bufset), C.c_int32, _P(ms_measure_cfg), C.c_void_p, _P(ms_measure_result)]),
    "ms_search_cfg_default": (None, [_P(ms_search_cfg)]),
    "ms_search": (C.c_int32, [C.c_void_p, _P(ms_space), _P(ms_search_cfg), _P(ms_bufset), C.c_int32, C.c_void_p,
                              LATENCY_FN, C.c_void_p, TRIAL_CB, C.c_void_p, _P(ms_search_result)]),
    "ms_device_info_get": (C.c_int32, [_P(ms_device_info)]),
    "ms_calibrate_mfma": (C.c_int32, [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, _P(C.c_double)]),
    "ms_calibrate_stream": (C.c_int32, [C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, _P(C.c_double)]),
    "ms_calibrate_lds": (C.c_int32, [C.c_void_p, C.c_void_p, _P(C.c_double), _P(C.c_double)]),
    "ms_calibrate_l2": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, _P(C.c_double)]),
    "ms_cost_model_create": (C.c_int32, [C.c_int32, C.c_int32, C.c_double, C.c_int32, _P(C.c_void_p)]),
    "ms_cost_model_destroy": (None, [C.c_void_p]),
    "ms_cost_model_fit": (C.c_int32, [C.c_void_p, _P(C.c_double), _P(C.c_double), C.c_int32, C.c_int32]),
    "ms_cost_model_predict": (C.c_int32, [C.c_void_p, _P(C.c_double), C.c_int32, C.c_int32, _P(C.c_double)]),
    "ms_variant_features": (C.c_int32, [C.c_void_p, _P(ms_variant_params), _P(C.c_double), C.c_int32, _P(C.c_int32)]),
    "ms_calibrate_timer": (C.c_int32, [C.c_double, _P(ms_measure_cfg), C.c_void_p, C.c_void_p, _P(ms_measure_result)]),
    "ms_version": (C.c_int32, []),
    "ms_last_error": (C.c_char_p, []),
}

_lib = None


def lib():
    """Load libms.so (built by build_lib.py / __graft_entry__.build()).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("%s is missing: run `python -m paper_2205_13603_amd.build_lib` (there is no fallback path)" % LIB_PATH)
        # PyTorch brings its own copy of the HIP runtime.  Loaded after libms.so's, it found no device on the MI355X
        # boxes ("no ROCm-capable device is detected" from the first HIP call of libms.so); loaded first, both work.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def last_error():
    return lib().ms_last_error().decode("utf-8", "replace")


def _check(rc):
    if rc != MS_OK:
        raise MsError(rc, last_error())


# ------------------------------------------------------------------ thin object wrappers
class Op:
    def __init__(self, kind, in_dtype, out_dtype, dims, stride=0, pad=0, has_bias=False, relu=False,
                 a_strides=None, b_strides=None, dilation=0):
        d = ms_op_desc()
        d.kind = kind
        d.in_dtype = DTYPE_NAMES.get(in_dtype, in_dtype)
        d.out_dtype = DTYPE_NAMES.get(out_dtype, out_dtype)
        d.stride, d.pad, d.has_bias, d.relu, d.dilation = stride, pad, int(has_bias), int(relu), dilation
        for i, v in enumerate(dims):
            d.dims[i] = v
        for i, v in enumerate(a_strides or ()):
            d.a_strides[i] = v
        for i, v in enumerate(b_strides or ()):
            d.b_strides[i] = v
        self.handle = C.c_void_p()
        _check(lib().ms_op_create(C.byref(d), C.byref(self.handle)))

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ms_op_destroy(self.handle)
            self.handle = None

    def desc(self):
        d = ms_op_desc()
        _check(lib().ms_op_get_desc(self.handle, C.byref(d)))
        return d

    def loops(self):
        arr = (ms_loop * MAX_LOOPS)()
        n = C.c_int32()
        _check(lib().ms_op_loops(self.handle, arr, C.byref(n)))
        return [(arr[i].name.decode(), int(arr[i].extent), bool(arr[i].is_reduction)) for i in range(n.value)]

    def work(self):
        f, b = C.c_double(), C.c_double()
        _check(lib().ms_op_work(self.handle, C.byref(f), C.byref(b)))
        return f.value, b.value

    def tensor_bytes(self, idx):
        v = C.c_int64()
        _check(lib().ms_op_tensor_bytes(self.handle, idx, C.byref(v)))
        return v.value

    def space(self, flags=SPACE_DEFAULT):
        sp = ms_space()
        _check(lib().ms_space_describe(self.handle, flags, C.byref(sp)))
        return sp


def gemm_op(M, N, K, in_dtype="f32", out_dtype=None, **kw):
    return Op(OP_GEMM, in_dtype, out_dtype or ("i32" if in_dtype == "i8" else in_dtype), [M, N, K], **kw)


def bmm_op(B, M, N, K, trans_b, in_dtype="f16", out_dtype=None, **kw):
    return Op(OP_BMM_NT if trans_b else OP_BMM_NN, in_dtype, out_dtype or ("i32" if in_dtype == "i8" else in_dtype),
              [B, M, N, K], **kw)


def conv2d_op(N, H, W, Cin, Cout, KH, KW, stride=1, pad=0, has_bias=True, relu=True, in_dtype="f16", out_dtype=None, dilation=1,
              groups=1):
    """groups > 1: W is [KH][KW][Cin/groups][Cout] and an output channel sees the input channels of its own group."""
    return Op(OP_CONV2D_NHWC, in_dtype, out_dtype or in_dtype, [N, H, W, Cin, Cout, KH, KW] + ([groups] if groups > 1 else []), stride=stride, pad=pad,
              has_bias=has_bias, relu=relu, dilation=dilation)


def conv3d_op(N, D, H, W, Cin, Cout, K, stride=1, pad=0, has_bias=True, relu=True, in_dtype="f16", out_dtype=None, dilation=1):
    """3-D convolution with a K x K x K filter: X [N, D, H, W, Cin], W [K, K, K, Cin, Cout], Y [N, OD, OH, OW, Cout]."""
    return Op(OP_CONV3D_NDHWC, in_dtype, out_dtype or in_dtype, [N, D, H, W, Cin, Cout, K], stride=stride, pad=pad,
              has_bias=has_bias, relu=relu, dilation=dilation)


def conv1d_op(N, L, Cin, Cout, K, stride=1, pad=0, has_bias=True, relu=True, in_dtype="f16", out_dtype=None, dilation=1, groups=1):
    """1-D convolution: X [N, L, Cin], W [K, Cin/groups, Cout], Y [N, OL, Cout]; `pad` zeros at both ends of L."""
    return Op(OP_CONV1D_NWC, in_dtype, out_dtype or in_dtype, [N, L, Cin, Cout, K] + ([groups] if groups > 1 else []), stride=stride, pad=pad,
              has_bias=has_bias, relu=relu, dilation=dilation)


def conv2d_transposed_op(N, H, W, Cin, Cout, KH, KW, stride=1, pad=0, has_bias=True, relu=True, in_dtype="f16", out_dtype=None):
    """Transposed convolution: output [N, (H-1)*stride - 2*pad + KH, (W-1)*stride - 2*pad + KW, Cout]."""
    return Op(OP_CONV2D_TRANSPOSED_NHWC, in_dtype, out_dtype or in_dtype, [N, H, W, Cin, Cout, KH, KW], stride=stride, pad=pad,
              has_bias=has_bias, relu=relu, dilation=1)


def dwconv2d_op(N, H, W, Cc, KH=3, KW=3, stride=1, pad=1):
    return Op(OP_DWCONV2D_NHWC, "f32", "f32", [N, H, W, Cc, KH, KW], stride=stride, pad=pad)


def softmax_op(B, M, N, in_dtype="f32", out_dtype=None):
    """Softmax over the last axis of X [B, M, N]."""
    return Op(OP_SOFTMAX, in_dtype, out_dtype or in_dtype, [B, M, N])


def norm_op(B, M, N, in_dtype="f32"):
    """2-norm of each batch entry of X [B, M, N]; fp32 [B]."""
    return Op(OP_NORM, in_dtype, "f32", [B, M, N])


MAX_MODULES = 16


def modules():
    """The module table: list of dicts {index, name, primitives, location, flag, requires}."""
    out = []
    for i in range(lib().ms_module_count()):
        m = ms_module_info()
        _check(lib().ms_module_get(i, C.byref(m)))
        out.append({"index": i, "name": m.name.decode(), "primitives": m.primitives.decode(), "location": m.location,
                    "flag": m.flag, "requires": m.requires})
    return out


def module_indices(names):
    table = {m["name"]: m["index"] for m in modules()}
    return [table[n] if isinstance(n, str) else int(n) for n in names]


def space_compose(op, names_or_indices):
    """Compose(modules, e0): the space of an ordered module list; returns (space, applied mask)."""
    idx = module_indices(names_or_indices)
    arr = (C.c_int32 * len(idx))(*idx)
    sp, mask = ms_space(), C.c_uint32()
    _check(lib().ms_space_compose(op.handle, arr, len(idx), C.byref(mask), C.byref(sp)))
    return sp, mask.value


def space_stochastic_compose(op, names_or_indices, seed):
    """Stochastic-Compose over a module set; returns (space, names of the modules in the order they were applied)."""
    idx = module_indices(names_or_indices)
    arr = (C.c_int32 * max(1, len(idx)))(*idx)
    applied, n = (C.c_int32 * MAX_MODULES)(), C.c_int32()
    sp = ms_space()
    _check(lib().ms_space_stochastic_compose(op.handle, arr, len(idx), seed, applied, C.byref(n), C.byref(sp)))
    names = {m["index"]: m["name"] for m in modules()}
    return sp, [names[applied[i]] for i in range(n.value)]


def space_log10_size(space):
    v = C.c_double()
    _check(lib().ms_space_log10_size(C.byref(space), C.byref(v)))
    return v.value


def trace_sample(space, seed, index):
    t = ms_trace()
    _check(lib().ms_trace_sample(C.byref(space), seed, index, C.byref(t)))
    return t


def trace_sample_valid(op, space, seed, index, max_tries=1000):
    t = ms_trace()
    _check(lib().ms_trace_sample_valid(op.handle, C.byref(space), seed, index, max_tries, C.byref(t)))
    return t


def trace_mutate(space, trace, seed):
    t = ms_trace()
    _check(lib().ms_trace_mutate(C.byref(space), C.byref(trace), seed, C.byref(t)))
    return t


def trace_to_text(op, space, trace):
    need = C.c_size_t()
    _check(lib().ms_trace_to_text(op.handle, C.byref(space), C.byref(trace), None, 0, C.byref(need)))
    buf = C.create_string_buffer(need.value)
    _check(lib().ms_trace_to_text(op.handle, C.byref(space), C.byref(trace), buf, need.value, None))
    return buf.value.decode()


def trace_from_text(space, text):
    t = ms_trace()
    _check(lib().ms_trace_from_text(C.byref(space), text.encode(), C.byref(t)))
    return t


def trace_validate(op, space, trace):
    p = ms_variant_params()
    _check(lib().ms_trace_validate(op.handle, C.byref(space), C.byref(trace), C.byref(p)))
    return p


def make_trace(space, values):
    """Build a trace from plain lists: one list per slot (tile factors, or [candidate value])."""
    t = ms_trace()
    t.n = space.n_slots
    assert len(values) == space.n_slots
    for i, vals in enumerate(values):
        s = space.slots[i]
        t.d[i].slot_id, t.d[i].kind = s.slot_id, s.kind
        if s.kind == SLOT_CATEGORICAL:
            cands = [s.candidates[c] for c in range(s.n_candidates)]
            (val,) = vals if isinstance(vals, (list, tuple)) else (vals,)
            t.d[i].n = 1
            t.d[i].v[0] = cands.index(val)
        else:
            t.d[i].n = len(vals)
            for k, v in enumerate(vals):
                t.d[i].v[k] = v
    return t


def trace_from_decisions(space, decisions):
    """Inverse of ms_trace.decisions(): [(slot_id, [raw values])] in the space's slot order -> trace."""
    if len(decisions) != space.n_slots:
        raise ValueError("%d decisions for a space of %d slots" % (len(decisions), space.n_slots))
    t = ms_trace()
    t.n = space.n_slots
    for i, (slot_id, vals) in enumerate(decisions):
        s = space.slots[i]
        if s.slot_id != slot_id:
            raise ValueError("decision %d is for slot %d, the space has slot %d there" % (i, slot_id, s.slot_id))
        t.d[i].slot_id, t.d[i].kind, t.d[i].n = s.slot_id, s.kind, len(vals)
        for k, v in enumerate(vals):
            t.d[i].v[k] = v
    return t


def get_limits():
    lim = ms_limits()
    _check(lib().ms_get_limits(C.byref(lim)))
    return lim


def set_limits(lim):
    _check(lib().ms_set_limits(C.byref(lim)))


def variant_coverage(op, params, out_elems):
    import numpy as np
    counts = np.zeros(out_elems, np.int32)
    _check(lib().ms_variant_coverage(op.handle, C.byref(params), counts.ctypes.data_as(C.c_void_p), out_elems))
    return counts


def variant_reduction_coverage(op, params):
    import numpy as np
    need = C.c_int64()
    _check(lib().ms_variant_reduction_coverage(op.handle, C.byref(params), None, 0, C.byref(need)))
    counts = np.zeros(need.value, np.int32)
    _check(lib().ms_variant_reduction_coverage(op.handle, C.byref(params), counts.ctypes.data_as(C.c_void_p), need.value, None))
    return counts


def variant_kernel_text(op, params):
    need = C.c_size_t()
    _check(lib().ms_variant_kernel_text(op.handle, C.byref(params), None, 0, C.byref(need)))
    buf = C.create_string_buffer(need.value)
    _check(lib().ms_variant_kernel_text(op.handle, C.byref(params), buf, need.value, None))
    return buf.value.decode()


def prebuild(op, space, traces, threads=8):
    arr = (ms_trace * len(traces))(*traces)
    n = C.c_int32()
    _check(lib().ms_prebuild(op.handle, C.byref(space), arr, len(traces), threads, C.byref(n)))
    return n.value


def set_cache_dir(path):
    _check(lib().ms_set_cache_dir(path.encode() if path else None))


def _bufsets(bufsets):
    """[(inputs, output[, workspace])] of device pointers -> array of ms_bufset (at least one element)."""
    arr = (ms_bufset * max(1, len(bufsets)))()
    for i, bs in enumerate(bufsets):
        for k, p in enumerate(bs[0]):
            arr[i].inputs[k] = p
        arr[i].output = bs[1]
        arr[i].workspace = bs[2] if len(bs) > 2 else None
    return arr


def jit_stats():
    """{compiled, from_disk, from_memory, compiler: (major, minor)} of this process."""
    a, b, c, mj, mn = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int32(), C.c_int32()
    _check(lib().ms_jit_stats(C.byref(a), C.byref(b), C.byref(c), C.byref(mj), C.byref(mn)))
    return {"compiled": a.value, "from_disk": b.value, "from_memory": c.value, "compiler": (mj.value, mn.value)}


class Variant:
    def __init__(self, op, space, trace):
        self.op = op
        self.handle = C.c_void_p()
        _check(lib().ms_variant_build(op.handle, C.byref(space), C.byref(trace), C.byref(self.handle)))

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ms_variant_destroy(self.handle)
            self.handle = None

    def params(self):
        p = ms_variant_params()
        ws = C.c_size_t()
        _check(lib().ms_variant_info(self.handle, C.byref(p), C.byref(ws)))
        return p

    def resources(self):
        """Registers, scratch and LDS of the compiled kernel, from its code object's metadata."""
        r = ms_variant_resources()
        _check(lib().ms_variant_resources_get(self.handle, C.byref(r)))
        return r

    def workspace_bytes(self):
        """Bytes of workspace one instance needs (0 unless the reduction is split across workgroups);
        a launch over R instances takes R times as much."""
        ws = C.c_size_t()
        _check(lib().ms_variant_info(self.handle, None, C.byref(ws)))
        return ws.value

    def launch(self, inputs, output, instances=1, stream=None, workspace=None):
        """inputs / output / workspace: device pointers (ints)."""
        ins = (C.c_void_p * 4)(*[C.c_void_p(p) for p in inputs])
        outs = (C.c_void_p * 1)(C.c_void_p(output))
        _check(lib().ms_variant_launch(self.handle, ins, outs, workspace, instances, stream))

    def prepare(self):
        """Set-up for launch_static: loads the kernels on the current device, resolves the built-in workspace."""
        _check(lib().ms_variant_prepare(self.handle))

    def launch_static(self, inputs, output, instances=1, stream=None):
        """launch() with the workspace taken from the library's built-in array; allocates nothing."""
        ins = (C.c_void_p * 4)(*[C.c_void_p(p) for p in inputs])
        outs = (C.c_void_p * 1)(C.c_void_p(output))
        _check(lib().ms_variant_launch_static(self.handle, ins, outs, instances, stream))

    def measure(self, bufsets, warmup=2, repeats=5, launches_per_repeat=20, instances=1, stream=None):
        """bufsets: list of (inputs, output) or (inputs, output, workspace) device pointer tuples."""
        arr = _bufsets(bufsets)
        cfg = ms_measure_cfg(warmup, repeats, launches_per_repeat, instances)
        res = ms_measure_result()
        _check(lib().ms_measure(self.handle, arr, len(bufsets), C.byref(cfg), stream, C.byref(res)))
        return res


def device_info():
    info = ms_device_info()
    _check(lib().ms_device_info_get(C.byref(info)))
    return info


def calibrate_mfma(in_dtype, mfma_code, scratch_ptr, operands_ptr=None, stream=None):
    v = C.c_double()
    _check(lib().ms_calibrate_mfma(DTYPE_NAMES.get(in_dtype, in_dtype), mfma_code, operands_ptr, scratch_ptr, stream, C.byref(v)))
    return v.value


def calibrate_stream(mode, src_ptr, dst_ptr, nbytes, stream=None):
    v = C.c_double()
    _check(lib().ms_calibrate_stream(mode, src_ptr, dst_ptr, nbytes, stream, C.byref(v)))
    return v.value


def calibrate_lds(scratch_ptr, stream=None):
    a, b = C.c_double(), C.c_double()
    _check(lib().ms_calibrate_lds(scratch_ptr, stream, C.byref(a), C.byref(b)))
    return a.value, b.value


def calibrate_l2(src_ptr, scratch_ptr, stream=None):
    v = C.c_double()
    _check(lib().ms_calibrate_l2(src_ptr, scratch_ptr, stream, C.byref(v)))
    return v.value


def calibrate_timer(target_us, scratch_ptr, warmup=2, repeats=5, launches_per_repeat=1, stream=None):
    cfg = ms_measure_cfg(warmup, repeats, launches_per_repeat, 1)
    res = ms_measure_result()
    _check(lib().ms_calibrate_timer(target_us, C.byref(cfg), scratch_ptr, stream, C.byref(res)))
    return res


class CostModel:
    """Gradient-boosted regression trees of the library (fit / predict on numpy float64 arrays)."""

    def __init__(self, n_trees=50, depth=3, learning_rate=0.3, min_leaf=2):
        self.handle = C.c_void_p()
        _check(lib().ms_cost_model_create(n_trees, depth, learning_rate, min_leaf, C.byref(self.handle)))

    def __del__(self):
        if getattr(self, "handle", None):
            lib().ms_cost_model_destroy(self.handle)
            self.handle = None

    def fit(self, X, y):
        import numpy as np
        X = np.ascontiguousarray(X, dtype=np.float64)
        y = np.ascontiguousarray(y, dtype=np.float64)
        n, d = X.shape
        assert y.shape == (n,)
        _check(lib().ms_cost_model_fit(self.handle, X.ctypes.data_as(_P(C.c_double)), y.ctypes.data_as(_P(C.c_double)), n, d))

    def predict(self, X):
        import numpy as np
        X = np.ascontiguousarray(X, dtype=np.float64)
        n, d = X.shape
        out = np.empty(n, dtype=np.float64)
        _check(lib().ms_cost_model_predict(self.handle, X.ctypes.data_as(_P(C.c_double)), n, d, out.ctypes.data_as(_P(C.c_double))))
        return out


def variant_features(op, params):
    import numpy as np
    n = C.c_int32()
    _check(lib().ms_variant_features(op.handle, C.byref(params), None, 0, C.byref(n)))
    out = np.empty(n.value, dtype=np.float64)
    _check(lib().ms_variant_features(op.handle, C.byref(params), out.ctypes.data_as(_P(C.c_double)), n.value, C.byref(n)))
    return out


def search_cfg_default():
    cfg = ms_search_cfg()
    lib().ms_search_cfg_default(C.byref(cfg))
    return cfg


def search(op, space, cfg, bufsets=(), stream=None, fake_latency=None, on_trial=None, pretrain=None):
    """pretrain = (X, y): rows for cfg.pretrain_X / pretrain_y (features as variant_features gives them, log2 microseconds)."""
    arr = _bufsets(bufsets)
    if pretrain is not None:
        import numpy as np
        X = np.ascontiguousarray(pretrain[0], dtype=np.float64)
        y = np.ascontiguousarray(pretrain[1], dtype=np.float64)
        if X.ndim != 2 or y.shape != (X.shape[0],):
            raise ValueError("pretrain: X must be n x d and y of length n")
        cfg.pretrain_n, cfg.pretrain_d = X.shape
        cfg.pretrain_X = X.ctypes.data_as(C.POINTER(C.c_double))
        cfg.pretrain_y = y.ctypes.data_as(C.POINTER(C.c_double))
    res = ms_search_result()
    lat = LATENCY_FN(lambda p, u: float(fake_latency(p.contents))) if fake_latency else C.cast(None, LATENCY_FN)
    cb = TRIAL_CB(lambda t, u: int(on_trial(t.contents) or 0)) if on_trial else C.cast(None, TRIAL_CB)
    try:
        _check(lib().ms_search(op.handle, C.byref(space), C.byref(cfg), arr, len(bufsets), stream, lat, None, cb, None,
                               C.byref(res)))
    finally:
        if pretrain is not None:  # the arrays live only as long as this call
            cfg.pretrain_n = cfg.pretrain_d = 0
            cfg.pretrain_X = cfg.pretrain_y = None
    return res
