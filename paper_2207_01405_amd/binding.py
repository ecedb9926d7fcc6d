"""Thin ctypes binding over the C ABI of libivit.so (see include/ivit.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels.  Functions carry the
names of the C entry points; tensors are torch CUDA tensors (device memory and streams are all torch
is used for).  There is no CPU path: loading fails loudly if the library has not been built.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_DEFAULT_LIB = os.path.join(_HERE, "libivit.so")
LIB_PATH = _DEFAULT_LIB     # tests of build variants may point this elsewhere before load()

IVIT_OK = 0
IVIT_ERR_NULL, IVIT_ERR_SHAPE, IVIT_ERR_PARAM, IVIT_ERR_ALIGN, IVIT_ERR_WORKSPACE, IVIT_ERR_HIP = -1, -2, -3, -4, -5, -6
ERRORS = {"NULL": -1, "SHAPE": -2, "PARAM": -3, "ALIGN": -4, "WORKSPACE": -5, "HIP": -6}

EXPORTS = ("ivit_strerror", "ivit_build_id", "ivit_linear_requant", "ivit_shiftmax", "ivit_shiftgelu", "ivit_shiftgelu_raw",
           "ivit_ilayernorm", "ivit_workspace_bytes", "ivit_attention", "ivit_encoder_block", "ivit_forward",
           "ivit_trace_begin", "ivit_trace_end", "ivit_quantize_symmetric", "ivit_dyadic_from_float",
           "ivit_shift_params_from_scale", "ivit_embed_tokens", "ivit_classifier_head", "ivit_image_workspace_bytes",
           "ivit_forward_image", "ivit_attention_masked", "ivit_window_attention", "ivit_window_attention_ex", "ivit_patch_merge_gather",
           "ivit_mean_pool", "ivit_swin_window_index", "ivit_swin_shift_mask", "ivit_swin_workspace_bytes",
           "ivit_forward_swin", "ivit_shiftgelu_rowmax", "ivit_encoder_block_static", "ivit_linear_requant_ex",
           "ivit_last_hip_error", "ivit_probe_mfma_rate", "ivit_ilayernorm_limits")

KIND_NAMES = {1: "ilayernorm", 2: "gemm", 3: "gemm_residual", 4: "gemm_gelu", 5: "attention", 6: "shiftmax",
              7: "shiftgelu", 8: "embed_tokens", 9: "patch_merge_gather", 10: "mean_pool"}


class ShiftParams(C.Structure):
    _fields_ = [("i0", C.c_int32), ("n_shift", C.c_int32), ("m_bits", C.c_int32), ("k_out", C.c_int32)]


class Dyadic(C.Structure):
    _fields_ = [("b", C.c_int32), ("c", C.c_int32)]


class LinearOptions(C.Structure):
    _fields_ = [("kernel", C.c_int32), ("rounding", C.c_int32)]


class AttentionOptions(C.Structure):
    _fields_ = [("rounding", C.c_int32)]


KERNELS = {"auto": 0, "many_rows": 1, "reg_stationary": 2, "big_tiles": 3}
ROUNDING = {"nearest": 0, "floor": 1}


class Dims(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "T", "C", "H", "F")]


_P = C.c_void_p


class BlockParams(C.Structure):
    _fields_ = [
        ("ln1_gamma", _P), ("ln1_beta", _P), ("ln1_f_bits", C.c_int32), ("ln1_c_shift", C.c_int32),
        ("w_qkv", _P), ("bias_qkv", _P), ("qkv_rq_b", _P), ("qkv_rq_c", _P),
        ("qk_rq", Dyadic), ("rel_bias", _P), ("softmax", ShiftParams), ("pv_rq", Dyadic),
        ("w_proj", _P), ("bias_proj", _P), ("proj_rq_b", _P), ("proj_rq_c", _P), ("res1_rq", Dyadic),
        ("ln2_gamma", _P), ("ln2_beta", _P), ("ln2_f_bits", C.c_int32), ("ln2_c_shift", C.c_int32),
        ("w_fc1", _P), ("bias_fc1", _P), ("fc1_rq_b", _P), ("fc1_rq_c", _P),
        ("gelu", ShiftParams), ("gelu_rq", Dyadic),
        ("w_fc2", _P), ("bias_fc2", _P), ("fc2_rq_b", _P), ("fc2_rq_c", _P), ("res2_rq", Dyadic),
        ("attn_mask", _P), ("n_mask", C.c_int32), ("tok_index", _P), ("n_win", C.c_int32),
    ]


TAP_NAMES = ("u", "qkv", "scores", "probs", "o", "xhat", "v", "h")


class DebugTaps(C.Structure):
    _fields_ = [(n, _P) for n in TAP_NAMES]


class ImageParams(C.Structure):
    _fields_ = [("w_patch", _P), ("bias_patch", _P), ("patch_rq_b", _P), ("patch_rq_c", _P), ("patch_dim", C.c_int32),
                ("cls", _P), ("pos", _P), ("tok_rq", Dyadic), ("pos_rq", Dyadic),
                ("w_head", _P), ("bias_head", _P), ("head_rq_b", _P), ("head_rq_c", _P), ("n_classes", C.c_int32)]


class FinalLN(C.Structure):
    _fields_ = [("gamma", _P), ("beta", _P), ("f_bits", C.c_int32), ("c_shift", C.c_int32)]


class SwinStage(C.Structure):
    _fields_ = [("C", C.c_int32), ("H", C.c_int32), ("F", C.c_int32), ("n_blocks", C.c_int32),
                ("blocks", C.POINTER(BlockParams)), ("merge_ln", FinalLN), ("w_merge", _P), ("merge_rq_b", _P),
                ("merge_rq_c", _P)]


class SwinParams(C.Structure):
    _fields_ = [("grid", C.c_int32), ("window", C.c_int32), ("n_stages", C.c_int32), ("patch_dim", C.c_int32),
                ("n_classes", C.c_int32), ("w_patch", _P), ("bias_patch", _P), ("patch_rq_b", _P), ("patch_rq_c", _P),
                ("embed_ln", FinalLN), ("stages", SwinStage * 4), ("final_ln", FinalLN), ("pool_rq", Dyadic),
                ("w_head", _P), ("bias_head", _P), ("head_rq_b", _P), ("head_rq_c", _P)]


class IvitError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, strerror(status), status))


_lib = None


def load():
    """Load libivit.so.  Raises if it is missing: build it with `python -m paper_2207_01405_amd.build`."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libivit.so is not built (%s); run `python -m paper_2207_01405_amd.build`" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    i32, i64 = C.c_int32, C.c_int64
    # a library built from other sources than the ones next to this file (a failed or forgotten rebuild) is refused
    lib.ivit_build_id.restype = C.c_char_p; lib.ivit_build_id.argtypes = []
    if LIB_PATH == _DEFAULT_LIB and os.path.isdir(os.path.join(_HERE, "csrc")):
        from . import build as _build
        have, want = lib.ivit_build_id().decode(), _build.source_id()
        if have != want:
            raise RuntimeError("libivit.so (build id %s) was not built from the present sources (%s); "
                               "run `python -m paper_2207_01405_amd.build`" % (have, want))
    lib.ivit_strerror.restype = C.c_char_p; lib.ivit_strerror.argtypes = [C.c_int]
    lib.ivit_linear_requant.restype = C.c_int
    lib.ivit_linear_requant.argtypes = [_P, _P, _P, _P, _P, _P, _P, Dyadic, C.POINTER(ShiftParams), Dyadic, _P, i64, i32, i32]
    lib.ivit_linear_requant_ex.restype = C.c_int
    lib.ivit_linear_requant_ex.argtypes = lib.ivit_linear_requant.argtypes + [C.POINTER(LinearOptions)]
    lib.ivit_last_hip_error.restype = C.c_int; lib.ivit_last_hip_error.argtypes = []
    lib.ivit_ilayernorm_limits.restype = C.c_int
    lib.ivit_ilayernorm_limits.argtypes = [i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.ivit_probe_mfma_rate.restype = C.c_int
    lib.ivit_probe_mfma_rate.argtypes = [_P, i32, i32, _P, C.c_size_t, C.POINTER(i64)]
    lib.ivit_shiftmax.restype = C.c_int
    lib.ivit_shiftmax.argtypes = [_P, _P, _P, i32, i32, _P, i64, i32, i32, ShiftParams]
    lib.ivit_shiftgelu.restype = C.c_int; lib.ivit_shiftgelu.argtypes = [_P, _P, _P, i64, ShiftParams, Dyadic]
    lib.ivit_shiftgelu_rowmax.restype = C.c_int; lib.ivit_shiftgelu_rowmax.argtypes = [_P, _P, _P, i64, i32, ShiftParams, Dyadic]
    lib.ivit_shiftgelu_raw.restype = C.c_int; lib.ivit_shiftgelu_raw.argtypes = [_P, _P, _P, i64, ShiftParams]
    lib.ivit_ilayernorm.restype = C.c_int; lib.ivit_ilayernorm.argtypes = [_P, _P, _P, _P, _P, i64, i32, i32, i32]
    lib.ivit_workspace_bytes.restype = C.c_size_t; lib.ivit_workspace_bytes.argtypes = [C.POINTER(Dims)]
    lib.ivit_attention.restype = C.c_int
    lib.ivit_attention.argtypes = [_P, _P, _P, _P, C.POINTER(Dims), Dyadic, ShiftParams, Dyadic, _P, _P]
    lib.ivit_attention_masked.restype = C.c_int
    lib.ivit_attention_masked.argtypes = [_P, _P, _P, _P, i32, _P, C.POINTER(Dims), Dyadic, ShiftParams, Dyadic, _P, _P]
    lib.ivit_window_attention.restype = C.c_int
    lib.ivit_window_attention.argtypes = [_P, _P, _P, _P, i32, _P, i32, _P, C.POINTER(Dims), Dyadic, ShiftParams, Dyadic, _P, _P]
    lib.ivit_window_attention_ex.restype = C.c_int
    lib.ivit_window_attention_ex.argtypes = lib.ivit_window_attention.argtypes + [C.POINTER(AttentionOptions)]
    lib.ivit_patch_merge_gather.restype = C.c_int; lib.ivit_patch_merge_gather.argtypes = [_P, _P, _P, i32, i32, i32]
    lib.ivit_mean_pool.restype = C.c_int; lib.ivit_mean_pool.argtypes = [_P, _P, _P, i32, i32, i32, Dyadic]
    lib.ivit_swin_window_index.restype = C.c_int; lib.ivit_swin_window_index.argtypes = [i32, i32, i32, _P]
    lib.ivit_swin_shift_mask.restype = C.c_int; lib.ivit_swin_shift_mask.argtypes = [i32, i32, i32, _P]
    lib.ivit_swin_workspace_bytes.restype = C.c_size_t; lib.ivit_swin_workspace_bytes.argtypes = [C.POINTER(SwinParams), i32]
    lib.ivit_forward_swin.restype = C.c_int
    lib.ivit_forward_swin.argtypes = [_P, _P, _P, C.POINTER(SwinParams), i32, _P, C.c_size_t]
    lib.ivit_encoder_block.restype = C.c_int
    lib.ivit_encoder_block.argtypes = [_P, _P, _P, C.POINTER(BlockParams), C.POINTER(Dims), _P, C.c_size_t,
                                       C.POINTER(DebugTaps)]
    lib.ivit_encoder_block_static.restype = C.c_int
    lib.ivit_encoder_block_static.argtypes = [_P, _P, _P, C.POINTER(BlockParams), C.POINTER(Dims), C.POINTER(DebugTaps)]
    lib.ivit_forward.restype = C.c_int
    lib.ivit_forward.argtypes = [_P, _P, _P, C.POINTER(BlockParams), i32, C.POINTER(FinalLN), C.POINTER(Dims), _P,
                                 C.c_size_t]
    lib.ivit_embed_tokens.restype = C.c_int
    lib.ivit_embed_tokens.argtypes = [_P, _P, _P, _P, Dyadic, Dyadic, _P, i32, i32, i32]
    lib.ivit_classifier_head.restype = C.c_int
    lib.ivit_classifier_head.argtypes = [_P, _P, i32, _P, _P, _P, _P, _P, i32, i32, i32]
    lib.ivit_image_workspace_bytes.restype = C.c_size_t; lib.ivit_image_workspace_bytes.argtypes = [C.POINTER(Dims)]
    lib.ivit_forward_image.restype = C.c_int
    lib.ivit_forward_image.argtypes = [_P, _P, _P, C.POINTER(ImageParams), C.POINTER(BlockParams), i32, C.POINTER(FinalLN),
                                       C.POINTER(Dims), _P, C.c_size_t]
    lib.ivit_quantize_symmetric.restype = C.c_int
    lib.ivit_quantize_symmetric.argtypes = [_P, i64, C.c_float, i32, _P, C.POINTER(C.c_float)]
    lib.ivit_dyadic_from_float.restype = C.c_int
    lib.ivit_dyadic_from_float.argtypes = [C.c_double, i32, C.POINTER(Dyadic)]
    lib.ivit_shift_params_from_scale.restype = C.c_int
    lib.ivit_shift_params_from_scale.argtypes = [C.c_double, i32, i32, i32, C.POINTER(ShiftParams)]
    lib.ivit_trace_begin.restype = C.c_int; lib.ivit_trace_begin.argtypes = [i32]
    lib.ivit_trace_end.restype = C.c_int
    lib.ivit_trace_end.argtypes = [C.POINTER(C.c_float), C.POINTER(i32), C.POINTER(i64), C.POINTER(i64), i32,
                                   C.POINTER(i32)]
    _lib = lib
    return lib


def ivit_trace_begin(max_launches):
    _check(load().ivit_trace_begin(int(max_launches)), "ivit_trace_begin")


def ivit_trace_end(capacity):
    """Returns a list of (milliseconds, kind, ops, bytes), one per launch since ivit_trace_begin."""
    ms = (C.c_float * capacity)(); kind = (C.c_int32 * capacity)()
    ops = (C.c_int64 * capacity)(); nbytes = (C.c_int64 * capacity)()
    count = C.c_int32(0)
    _check(load().ivit_trace_end(ms, kind, ops, nbytes, capacity, C.byref(count)), "ivit_trace_end")
    n = min(capacity, count.value)
    return [(ms[i], kind[i], ops[i], nbytes[i]) for i in range(n)]


def ivit_probe_mfma_rate(random_operands, iters, scratch, stream=None):
    """Launches the MFMA-only loop; returns the integer operations of the launch (time it with events on the stream)."""
    ops = C.c_int64(0)
    _check(load().ivit_probe_mfma_rate(_stream(stream), int(bool(random_operands)), int(iters), _ptr(scratch),
                                       scratch.numel() * scratch.element_size(), C.byref(ops)), "ivit_probe_mfma_rate")
    return ops.value


def ivit_ilayernorm_limits(Cc, f_bits, c_shift):
    """Host helper: (gamma_max, beta_max) under which ivit_ilayernorm is exact for every possible row."""
    g, b = C.c_int32(0), C.c_int32(0)
    _check(load().ivit_ilayernorm_limits(int(Cc), int(f_bits), int(c_shift), C.byref(g), C.byref(b)), "ivit_ilayernorm_limits")
    return g.value, b.value


def ivit_quantize_symmetric(r, m, k=8):
    """Host helper: numpy float32 array -> (int8 array, scale)."""
    import numpy as np
    r = np.ascontiguousarray(r, np.float32)
    q = np.empty(r.shape, np.int8)
    scale = C.c_float(0)
    _check(load().ivit_quantize_symmetric(r.ctypes.data, r.size, float(m), int(k), q.ctypes.data, C.byref(scale)),
           "ivit_quantize_symmetric")
    return q, scale.value


def ivit_dyadic_from_float(x, bits=15):
    """Host helper: positive real multiplier -> (b, c)."""
    d = Dyadic(0, 0)
    _check(load().ivit_dyadic_from_float(float(x), int(bits), C.byref(d)), "ivit_dyadic_from_float")
    return d.b, d.c


def ivit_shift_params_from_scale(s, width=16, m_bits=31, k_out=8):
    """Host helper: input scale of Shiftmax / ShiftGELU -> dict(i0, n_shift, m_bits, k_out)."""
    p = ShiftParams(0, 0, 0, 0)
    _check(load().ivit_shift_params_from_scale(float(s), int(width), int(m_bits), int(k_out), C.byref(p)),
           "ivit_shift_params_from_scale")
    return dict(i0=p.i0, n_shift=p.n_shift, m_bits=p.m_bits, k_out=p.k_out)


def strerror(status):
    return load().ivit_strerror(int(status)).decode()


def _check(status, where):
    if status != IVIT_OK:
        raise IvitError(status, where)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def shift_params(p):
    return p if isinstance(p, ShiftParams) else ShiftParams(int(p["i0"]), int(p["n_shift"]), int(p["m_bits"]), int(p["k_out"]))


def dyadic(p):
    if p is None:
        return Dyadic(0, 0)
    return p if isinstance(p, Dyadic) else Dyadic(int(p[0]), int(p[1]))


def dims(d):
    return d if isinstance(d, Dims) else Dims(*(int(d[k]) for k in "BTCHF"))


# ------------------------------------------------------------------ entry points (same names as the C ABI)
def ivit_linear_requant(x, w, bias, rq_b, rq_c, y, residual=None, res_rq=None, gelu=None, gelu_rq=None, stream=None,
                        kernel=None, rounding=None):
    """kernel, rounding: both None -> ivit_linear_requant; otherwise ivit_linear_requant_ex with kernel "auto" /
    "many_rows" / "reg_stationary" and rounding "nearest" / "floor"."""
    M, K = x.shape
    N = w.shape[0]
    g = None if gelu is None else C.byref(shift_params(gelu))
    args = (_stream(stream), _ptr(x), _ptr(w), _ptr(bias), _ptr(rq_b), _ptr(rq_c), _ptr(residual), dyadic(res_rq), g,
            dyadic(gelu_rq), _ptr(y), M, N, K)
    if kernel is None and rounding is None:
        _check(load().ivit_linear_requant(*args), "ivit_linear_requant")
    else:
        opt = LinearOptions(KERNELS[kernel or "auto"], ROUNDING[rounding or "nearest"])
        _check(load().ivit_linear_requant_ex(*args, C.byref(opt)), "ivit_linear_requant_ex")
    return y


def ivit_shiftmax(x, y, p, bias=None, H=1, T=1, cols=None, stream=None):
    rows, ld = x.shape
    cols = ld if cols is None else cols
    st = load().ivit_shiftmax(_stream(stream), _ptr(x), _ptr(bias), H, T, _ptr(y), rows, cols, ld, shift_params(p))
    _check(st, "ivit_shiftmax")
    return y


def ivit_shiftgelu(x, y, p, out_rq, stream=None):
    st = load().ivit_shiftgelu(_stream(stream), _ptr(x), _ptr(y), x.numel(), shift_params(p), dyadic(out_rq))
    _check(st, "ivit_shiftgelu")
    return y


def ivit_shiftgelu_rowmax(x, y, p, out_rq, stream=None):
    rows, cols = x.shape
    st = load().ivit_shiftgelu_rowmax(_stream(stream), _ptr(x), _ptr(y), rows, cols, shift_params(p), dyadic(out_rq))
    _check(st, "ivit_shiftgelu_rowmax")
    return y


def ivit_shiftgelu_raw(x, y16, p, stream=None):
    st = load().ivit_shiftgelu_raw(_stream(stream), _ptr(x), _ptr(y16), x.numel(), shift_params(p))
    _check(st, "ivit_shiftgelu_raw")
    return y16


def ivit_ilayernorm(x, gamma_q, beta_q, y, f_bits, c_shift, stream=None):
    rows, Cc = x.shape
    st = load().ivit_ilayernorm(_stream(stream), _ptr(x), _ptr(gamma_q), _ptr(beta_q), _ptr(y), rows, Cc,
                                int(f_bits), int(c_shift))
    _check(st, "ivit_ilayernorm")
    return y


def ivit_workspace_bytes(d):
    return int(load().ivit_workspace_bytes(C.byref(dims(d))))


def ivit_attention(qkv, o, d, qk_rq, softmax, pv_rq, rel_bias=None, tap_scores=None, tap_probs=None, stream=None, mask=None):
    if mask is None:
        st = load().ivit_attention(_stream(stream), _ptr(qkv), _ptr(rel_bias), _ptr(o), C.byref(dims(d)), dyadic(qk_rq),
                                   shift_params(softmax), dyadic(pv_rq), _ptr(tap_scores), _ptr(tap_probs))
    else:
        st = load().ivit_attention_masked(_stream(stream), _ptr(qkv), _ptr(rel_bias), _ptr(mask), int(mask.shape[0]), _ptr(o),
                                          C.byref(dims(d)), dyadic(qk_rq), shift_params(softmax), dyadic(pv_rq),
                                          _ptr(tap_scores), _ptr(tap_probs))
    _check(st, "ivit_attention")
    return o


_PTR_FIELDS = ("ln1_gamma", "ln1_beta", "w_qkv", "bias_qkv", "qkv_rq_b", "qkv_rq_c", "rel_bias", "w_proj", "bias_proj",
               "proj_rq_b", "proj_rq_c", "ln2_gamma", "ln2_beta", "w_fc1", "bias_fc1", "fc1_rq_b", "fc1_rq_c", "w_fc2",
               "bias_fc2", "fc2_rq_b", "fc2_rq_c")
_INT_FIELDS = ("ln1_f_bits", "ln1_c_shift", "ln2_f_bits", "ln2_c_shift")
_DY_FIELDS = ("qk_rq", "pv_rq", "res1_rq", "gelu_rq", "res2_rq")
_SP_FIELDS = ("softmax", "gelu")


def block_params(p):
    """BlockParams struct from a dict whose tensor entries are torch CUDA tensors (kept alive by the caller)."""
    if isinstance(p, BlockParams):
        return p
    bp = BlockParams()
    for k in _PTR_FIELDS:
        setattr(bp, k, _ptr(p.get(k)))
    for k in _INT_FIELDS:
        setattr(bp, k, int(p[k]))
    for k in _DY_FIELDS:
        setattr(bp, k, dyadic(p[k]))
    for k in _SP_FIELDS:
        setattr(bp, k, shift_params(p[k]))
    m = p.get("attn_mask")
    bp.attn_mask = _ptr(m)
    bp.n_mask = 1 if m is None else int(m.shape[0])
    ti = p.get("tok_index")
    bp.tok_index = _ptr(ti)
    bp.n_win = 1 if ti is None else int(ti.shape[0])
    return bp


def to_device(p, device="cuda"):
    """Copy the numpy arrays of a parameter dict to the device (torch tensors); other entries are kept."""
    import numpy as np
    import torch
    return {k: (torch.from_numpy(np.ascontiguousarray(v)).to(device) if isinstance(v, np.ndarray) else v)
            for k, v in p.items()}


def ivit_encoder_block(x, y, p, d, workspace, taps=None, stream=None):
    tp = None
    if taps is not None:
        tp = C.byref(DebugTaps(*[_ptr(taps.get(n)) for n in TAP_NAMES]))
    bp = block_params(p)
    st = load().ivit_encoder_block(_stream(stream), _ptr(x), _ptr(y), C.byref(bp), C.byref(dims(d)),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), tp)
    _check(st, "ivit_encoder_block")
    return y


STATIC_SCRATCH_BYTES = 32 << 20     # IVIT_STATIC_SCRATCH_BYTES of include/ivit.h


def ivit_encoder_block_static(x, y, p, d, taps=None, stream=None):
    tp = None
    if taps is not None:
        tp = C.byref(DebugTaps(*[_ptr(taps.get(n)) for n in TAP_NAMES]))
    bp = block_params(p)
    st = load().ivit_encoder_block_static(_stream(stream), _ptr(x), _ptr(y), C.byref(bp), C.byref(dims(d)), tp)
    _check(st, "ivit_encoder_block_static")
    return y


def ivit_forward(x, y, blocks, d, workspace, final_ln=None, stream=None):
    # a ctypes array of BlockParams is taken as it is (marshalled once by the caller, e.g. outside a timed loop)
    arr = blocks if isinstance(blocks, C.Array) else (BlockParams * max(1, len(blocks)))(*[block_params(p) for p in blocks])
    fl = None
    if final_ln is not None:
        fl = C.byref(FinalLN(_ptr(final_ln["gamma"]), _ptr(final_ln["beta"]), int(final_ln["f_bits"]),
                             int(final_ln["c_shift"])))
    st = load().ivit_forward(_stream(stream), _ptr(x), _ptr(y), arr, len(blocks), fl, C.byref(dims(d)),
                             _ptr(workspace), workspace.numel() * workspace.element_size())
    _check(st, "ivit_forward")
    return y


def ivit_embed_tokens(patch_tok, cls, pos, tok_rq, pos_rq, tokens, B, P, stream=None):
    Cc = tokens.shape[-1]
    _check(load().ivit_embed_tokens(_stream(stream), _ptr(patch_tok), _ptr(cls), _ptr(pos), dyadic(tok_rq), dyadic(pos_rq),
                                    _ptr(tokens), int(B), int(P), int(Cc)), "ivit_embed_tokens")
    return tokens


def ivit_classifier_head(tokens, T, w, bias, rq_b, rq_c, logits, stream=None):
    B, N = logits.shape
    _check(load().ivit_classifier_head(_stream(stream), _ptr(tokens), int(T), _ptr(w), _ptr(bias), _ptr(rq_b), _ptr(rq_c),
                                       _ptr(logits), int(B), int(N), int(w.shape[1])), "ivit_classifier_head")
    return logits


def ivit_image_workspace_bytes(d):
    return load().ivit_image_workspace_bytes(C.byref(dims(d)))


def image_params(p):
    """ImageParams struct from a dict whose tensor entries are torch CUDA tensors (kept alive by the caller)."""
    ip = ImageParams()
    for k in ("w_patch", "bias_patch", "patch_rq_b", "patch_rq_c", "cls", "pos", "w_head", "bias_head", "head_rq_b", "head_rq_c"):
        setattr(ip, k, _ptr(p.get(k)))
    ip.patch_dim = int(p["w_patch"].shape[1]); ip.n_classes = int(p["w_head"].shape[0])
    ip.tok_rq = dyadic(p["tok_rq"]); ip.pos_rq = dyadic(p["pos_rq"])
    return ip


def ivit_forward_image(patches, logits, image, blocks, d, workspace, final_ln, stream=None):
    # a ctypes array of BlockParams is taken as it is (marshalled once by the caller, e.g. outside a timed loop)
    arr = blocks if isinstance(blocks, C.Array) else (BlockParams * max(1, len(blocks)))(*[block_params(p) for p in blocks])
    fl = FinalLN(_ptr(final_ln["gamma"]), _ptr(final_ln["beta"]), int(final_ln["f_bits"]), int(final_ln["c_shift"]))
    ip = image if isinstance(image, ImageParams) else image_params(image)
    st = load().ivit_forward_image(_stream(stream), _ptr(patches), _ptr(logits), C.byref(ip), arr, len(blocks), C.byref(fl),
                                   C.byref(dims(d)), _ptr(workspace), workspace.numel() * workspace.element_size())
    _check(st, "ivit_forward_image")
    return logits


def ivit_window_attention(qkv, o, d, qk_rq, softmax, pv_rq, rel_bias, tok_index, mask=None, tap_scores=None, tap_probs=None,
                          stream=None, rounding=None):
    """tok_index: None or int32 CUDA tensor [n_win, T]; mask: None or int8 [n_mask, T, T]; rounding: None (the entry point
    without options) or "nearest" / "floor" (ivit_window_attention_ex)."""
    args = (_stream(stream), _ptr(qkv), _ptr(rel_bias), _ptr(mask), 1 if mask is None else int(mask.shape[0]), _ptr(tok_index),
            1 if tok_index is None else int(tok_index.shape[0]), _ptr(o), C.byref(dims(d)), dyadic(qk_rq), shift_params(softmax),
            dyadic(pv_rq), _ptr(tap_scores), _ptr(tap_probs))
    if rounding is None:
        _check(load().ivit_window_attention(*args), "ivit_window_attention")
    else:
        _check(load().ivit_window_attention_ex(*args, C.byref(AttentionOptions(ROUNDING[rounding]))), "ivit_window_attention_ex")
    return o


def ivit_patch_merge_gather(x, y, B, g, Cc, stream=None):
    _check(load().ivit_patch_merge_gather(_stream(stream), _ptr(x), _ptr(y), int(B), int(g), int(Cc)), "ivit_patch_merge_gather")
    return y


def ivit_mean_pool(x, y, B, T, Cc, rq, stream=None):
    _check(load().ivit_mean_pool(_stream(stream), _ptr(x), _ptr(y), int(B), int(T), int(Cc), dyadic(rq)), "ivit_mean_pool")
    return y


def ivit_swin_window_index(g, window, shift):
    """Host helper: numpy int32 [(g / window)^2, window^2]."""
    import numpy as np
    out = np.empty(((g // max(window, 1)) ** 2 if window > 0 else 0, window * window), np.int32)
    _check(load().ivit_swin_window_index(int(g), int(window), int(shift), out.ctypes.data), "ivit_swin_window_index")
    return out


def ivit_swin_shift_mask(g, window, shift):
    """Host helper: numpy int8 [(g / window)^2, window^2, window^2]."""
    import numpy as np
    T = window * window
    out = np.empty(((g // max(window, 1)) ** 2 if window > 0 else 0, T, T), np.int8)
    _check(load().ivit_swin_shift_mask(int(g), int(window), int(shift), out.ctypes.data), "ivit_swin_shift_mask")
    return out


def swin_to_device(model, device="cuda"):
    """Uploads a windowed model (dict as the synthetic generator makes it) and attaches to every block the token-index
    table and, for shifted blocks, the mask of its stage, built by the library's host helpers."""
    import torch
    up = lambda a: torch.from_numpy(a).to(device)
    m = {k: v for k, v in model.items() if k not in ("embed", "stages", "final_ln", "head")}
    for k in ("embed", "final_ln", "head"):
        m[k] = to_device(model[k], device)
    m["stages"] = []
    tables = {}
    for st in model["stages"]:
        g, window = st["grid"], model["window"]
        blocks = []
        for p in st["blocks"]:
            q = to_device({k: v for k, v in p.items() if k != "shift"}, device)
            if g > window:
                key = (g, p["shift"])
                if key not in tables:
                    tables[key] = (up(ivit_swin_window_index(g, window, p["shift"])),
                                   up(ivit_swin_shift_mask(g, window, p["shift"])) if p["shift"] else None)
                q["tok_index"], q["attn_mask"] = tables[key]
            blocks.append(q)
        m["stages"].append(dict(C=st["C"], H=st["H"], grid=g, blocks=blocks,
                                merge=None if st["merge"] is None else to_device(st["merge"], device)))
    return m


def swin_params(m):
    """SwinParams struct from a device model (swin_to_device); returns (struct, keep-alive list)."""
    sp_ = SwinParams()
    keep = []
    sp_.grid, sp_.window, sp_.n_stages = int(m["grid"]), int(m["window"]), len(m["stages"])
    sp_.patch_dim, sp_.n_classes = int(m["patch_dim"]), int(m["n_classes"])
    e = m["embed"]
    sp_.w_patch, sp_.bias_patch, sp_.patch_rq_b, sp_.patch_rq_c = _ptr(e["w"]), _ptr(e["bias"]), _ptr(e["rq_b"]), _ptr(e["rq_c"])
    sp_.embed_ln = FinalLN(_ptr(e["ln_gamma"]), _ptr(e["ln_beta"]), int(e["f_bits"]), int(e["c_shift"]))
    for i, st in enumerate(m["stages"]):
        sg = sp_.stages[i]
        sg.C, sg.H, sg.F, sg.n_blocks = int(st["C"]), int(st["H"]), 4 * int(st["C"]), len(st["blocks"])
        arr = (BlockParams * max(1, len(st["blocks"])))(*[block_params(p) for p in st["blocks"]])
        keep.append(arr)
        sg.blocks = arr
        mg = st["merge"]
        if mg is not None:
            sg.merge_ln = FinalLN(_ptr(mg["ln_gamma"]), _ptr(mg["ln_beta"]), int(mg["f_bits"]), int(mg["c_shift"]))
            sg.w_merge, sg.merge_rq_b, sg.merge_rq_c = _ptr(mg["w"]), _ptr(mg["rq_b"]), _ptr(mg["rq_c"])
    f = m["final_ln"]
    sp_.final_ln = FinalLN(_ptr(f["gamma"]), _ptr(f["beta"]), int(f["f_bits"]), int(f["c_shift"]))
    sp_.pool_rq = dyadic(m["pool_rq"])
    h = m["head"]
    sp_.w_head, sp_.bias_head, sp_.head_rq_b, sp_.head_rq_c = _ptr(h["w"]), _ptr(h["bias"]), _ptr(h["rq_b"]), _ptr(h["rq_c"])
    return sp_, keep


def ivit_swin_workspace_bytes(params, B):
    return int(load().ivit_swin_workspace_bytes(C.byref(params), int(B)))


def ivit_forward_swin(patches, logits, params, B, workspace, stream=None):
    st = load().ivit_forward_swin(_stream(stream), _ptr(patches), _ptr(logits), C.byref(params), int(B), _ptr(workspace),
                                  workspace.numel() * workspace.element_size())
    _check(st, "ivit_forward_swin")
    return logits
