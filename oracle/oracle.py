"""ctypes front end of the CPU oracle (ivit_oracle.c).  TEST INFRASTRUCTURE ONLY.

Compiles the C file with gcc on first use (plain -O2, no threads) and exposes
numpy-in / numpy-out wrappers.  The integer operators live in the C file; this
module marshals arguments and, for the layers around the encoder (token
assembly, the window / stage structure of the windowed models, pooling), strings
those operators together with plain numpy reshapes and int64 arithmetic.  It
imports nothing from the GPU package.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ivit_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

__all__ = [
    "build", "rnd_shift", "clamp_k", "requant", "shiftexp", "intdiv", "isqrt10",
    "shiftgelu_raw", "shiftgelu", "shiftgelu_rowmax", "shiftmax", "ilayernorm", "linear_requant",
    "attention", "encoder_block", "forward", "ShiftParams", "Dyadic",
    "requant_vec", "rnd_shift_vec", "isqrt10_vec", "shiftexp_vec", "TAP_NAMES",
    "quantize_symmetric", "dyadic_from_float", "shift_params_from_scale",
    "embed_tokens", "classifier_head", "forward_image",
    "window_partition", "window_reverse", "shift_mask", "swin_block", "patch_merge", "mean_pool", "swin_forward",
]


class ShiftParams(C.Structure):
    _fields_ = [("i0", C.c_int32), ("n_shift", C.c_int32), ("m_bits", C.c_int32), ("k_out", C.c_int32)]


class Dyadic(C.Structure):
    _fields_ = [("b", C.c_int32), ("c", C.c_int32)]


class _Dims(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "T", "C", "H", "F")]


_P = C.c_void_p


class _BlockParams(C.Structure):
    _fields_ = [
        ("ln1_gamma", _P), ("ln1_beta", _P), ("ln1_f_bits", C.c_int32), ("ln1_c_shift", C.c_int32),
        ("w_qkv", _P), ("bias_qkv", _P), ("qkv_rq_b", _P), ("qkv_rq_c", _P),
        ("qk_rq", Dyadic), ("rel_bias", _P), ("softmax", ShiftParams), ("pv_rq", Dyadic),
        ("w_proj", _P), ("bias_proj", _P), ("proj_rq_b", _P), ("proj_rq_c", _P), ("res1_rq", Dyadic),
        ("ln2_gamma", _P), ("ln2_beta", _P), ("ln2_f_bits", C.c_int32), ("ln2_c_shift", C.c_int32),
        ("w_fc1", _P), ("bias_fc1", _P), ("fc1_rq_b", _P), ("fc1_rq_c", _P),
        ("gelu", ShiftParams), ("gelu_rq", Dyadic),
        ("w_fc2", _P), ("bias_fc2", _P), ("fc2_rq_b", _P), ("fc2_rq_c", _P), ("res2_rq", Dyadic),
        ("attn_mask", _P), ("n_mask", C.c_int32),
    ]


class _Taps(C.Structure):
    _fields_ = [(n, _P) for n in ("u", "qkv", "scores", "probs", "o", "xhat", "v", "h")]


def build(force=False):
    """Compile ivit_oracle.c into liboracle.so (gcc -O2).  Returns the path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fwrapv", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        i64, i32 = C.c_int64, C.c_int32
        lib.orc_rnd_shift.restype = i64; lib.orc_rnd_shift.argtypes = [i64, i32]
        lib.orc_clamp_k.restype = i64; lib.orc_clamp_k.argtypes = [i64, i32]
        lib.orc_requant.restype = i64; lib.orc_requant.argtypes = [i64, i32, i32]
        lib.orc_shiftexp.restype = i64; lib.orc_shiftexp.argtypes = [i64, i32, i32]
        lib.orc_intdiv.restype = i64; lib.orc_intdiv.argtypes = [i64, i64, i32, i32]
        lib.orc_isqrt10.restype = i64; lib.orc_isqrt10.argtypes = [i64]
        lib.orc_shiftgelu_raw.restype = None; lib.orc_shiftgelu_raw.argtypes = [_P, _P, i64, ShiftParams]
        lib.orc_shiftgelu.restype = None; lib.orc_shiftgelu.argtypes = [_P, _P, i64, ShiftParams, Dyadic]
        lib.orc_shiftgelu_rowmax.restype = None
        lib.orc_shiftgelu_rowmax.argtypes = [_P, _P, i64, i32, ShiftParams, Dyadic]
        lib.orc_shiftmax.restype = None
        lib.orc_shiftmax.argtypes = [_P, _P, i32, i32, _P, i64, i32, i32, ShiftParams]
        lib.orc_ilayernorm.restype = None; lib.orc_ilayernorm.argtypes = [_P, _P, _P, _P, i64, i32, i32, i32]
        lib.orc_linear_requant.restype = None
        lib.orc_linear_requant.argtypes = [_P, _P, _P, _P, _P, _P, Dyadic, C.POINTER(ShiftParams), Dyadic,
                                           _P, i64, i32, i32]
        lib.orc_linear_requant_mode.restype = None
        lib.orc_linear_requant_mode.argtypes = lib.orc_linear_requant.argtypes + [i32]
        lib.orc_attention_masked.restype = None
        lib.orc_attention_masked.argtypes = [_P, _P, _P, C.c_int32, _P, _Dims, Dyadic, ShiftParams, Dyadic, _P, _P]
        lib.orc_attention_mode.restype = None
        lib.orc_attention_mode.argtypes = lib.orc_attention_masked.argtypes + [i32]
        lib.orc_encoder_block.restype = None
        lib.orc_encoder_block.argtypes = [_P, _P, C.POINTER(_BlockParams), _Dims, C.POINTER(_Taps)]
        lib.orc_forward.restype = None
        lib.orc_forward.argtypes = [_P, _P, C.POINTER(_BlockParams), i32, _P, _P, i32, i32, _Dims]
        lib.orc_requant_vec.restype = None; lib.orc_requant_vec.argtypes = [_P, _P, i64, i32, i32]
        lib.orc_rnd_shift_vec.restype = None; lib.orc_rnd_shift_vec.argtypes = [_P, _P, i64, i32]
        lib.orc_isqrt10_vec.restype = None; lib.orc_isqrt10_vec.argtypes = [_P, _P, i64]
        lib.orc_shiftexp_vec.restype = None; lib.orc_shiftexp_vec.argtypes = [_P, _P, i64, i32, i32]
        _lib = lib
    return _lib


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_P)


def _sp(p):
    return p if isinstance(p, ShiftParams) else ShiftParams(int(p["i0"]), int(p["n_shift"]), int(p["m_bits"]), int(p["k_out"]))


def _dy(p):
    if p is None:
        return Dyadic(0, 0)
    return p if isinstance(p, Dyadic) else Dyadic(int(p[0]), int(p[1]))


# ------------------------------------------------------------------ scalars
def rnd_shift(v, c): return int(_L().orc_rnd_shift(int(v), int(c)))
def clamp_k(v, k): return int(_L().orc_clamp_k(int(v), int(k)))
def requant(v, b, c): return int(_L().orc_requant(int(v), int(b), int(c)))
def shiftexp(i, i0, n_shift): return int(_L().orc_shiftexp(int(i), int(i0), int(n_shift)))
def intdiv(i1, i2, k_out, m_bits): return int(_L().orc_intdiv(int(i1), int(i2), int(k_out), int(m_bits)))
def isqrt10(v): return int(_L().orc_isqrt10(int(v)))


def _vec(fn, v, *args):
    v = _arr(v, np.int64)
    out = np.empty_like(v)
    fn(_ptr(v), _ptr(out), v.size, *args)
    return out


def requant_vec(v, b, c): return _vec(_L().orc_requant_vec, v, int(b), int(c))
def rnd_shift_vec(v, c): return _vec(_L().orc_rnd_shift_vec, v, int(c))
def isqrt10_vec(v): return _vec(_L().orc_isqrt10_vec, v)
def shiftexp_vec(v, i0, n_shift): return _vec(_L().orc_shiftexp_vec, v, int(i0), int(n_shift))


# ------------------------------------------------------------------ tensors
def shiftgelu_raw(x, p):
    x = _arr(x, np.int8)
    g = np.empty(x.shape, np.int32)
    _L().orc_shiftgelu_raw(_ptr(x), _ptr(g), x.size, _sp(p))
    return g


def shiftgelu(x, p, out_rq):
    x = _arr(x, np.int8)
    y = np.empty(x.shape, np.int8)
    _L().orc_shiftgelu(_ptr(x), _ptr(y), x.size, _sp(p), _dy(out_rq))
    return y


def shiftgelu_rowmax(x, p, out_rq):
    """x: int8 [rows, cols]; the maximum of Algorithm 2 is taken over each row."""
    x = _arr(x, np.int8)
    rows, cols = x.shape
    y = np.empty_like(x)
    _L().orc_shiftgelu_rowmax(_ptr(x), _ptr(y), rows, cols, _sp(p), _dy(out_rq))
    return y


def shiftmax(x, p, bias=None, H=1, T=1, cols=None):
    """x: int8 [rows, ld]; the first `cols` entries of each row are used."""
    x = _arr(x, np.int8)
    rows, ld = x.shape
    cols = ld if cols is None else cols
    if bias is not None:
        bias = _arr(bias, np.int8)
    y = np.empty((rows, cols), np.int8)
    _L().orc_shiftmax(_ptr(x), _ptr(bias), int(H), int(T), _ptr(y), rows, cols, ld, _sp(p))
    return y


def ilayernorm(x, gamma_q, beta_q, f_bits, c_shift):
    x = _arr(x, np.int8)
    g = _arr(gamma_q, np.int32); b = _arr(beta_q, np.int32)
    rows, Cc = x.shape
    assert g.shape == (Cc,) and b.shape == (Cc,)
    y = np.empty_like(x)
    _L().orc_ilayernorm(_ptr(x), _ptr(g), _ptr(b), _ptr(y), rows, Cc, int(f_bits), int(c_shift))
    return y


def linear_requant(x, w, bias, rq_b, rq_c, residual=None, res_rq=None, gelu=None, gelu_rq=None, floor_shift=False):
    """floor_shift: every dyadic requantisation of the layer as the bare shift Eq. 10 prints instead of the rounded one."""
    x = _arr(x, np.int8); w = _arr(w, np.int8)
    M, K = x.shape
    N, K2 = w.shape
    assert K == K2
    bias = None if bias is None else _arr(bias, np.int32)
    rq_b = _arr(rq_b, np.int32); rq_c = _arr(rq_c, np.int32)
    assert rq_b.shape == (N,) and rq_c.shape == (N,)
    residual = None if residual is None else _arr(residual, np.int8)
    if residual is not None:
        assert residual.shape == (M, N)
    y = np.empty((M, N), np.int8)
    g = None if gelu is None else C.pointer(_sp(gelu))
    args = (_ptr(x), _ptr(w), _ptr(bias), _ptr(rq_b), _ptr(rq_c), _ptr(residual), _dy(res_rq), g, _dy(gelu_rq), _ptr(y), M, N, K)
    if floor_shift:
        _L().orc_linear_requant_mode(*args, 1)
    else:
        _L().orc_linear_requant(*args)
    return y


def _dims(d):
    return _Dims(int(d["B"]), int(d["T"]), int(d["C"]), int(d["H"]), int(d["F"]))


def attention(qkv, dims, qk_rq, softmax, pv_rq, rel_bias=None, want_taps=False, mask=None, floor_shift=False):
    """mask: None or int8 [n_mask, T, T]; window b uses mask[b % n_mask]; nonzero entries add -100 (real units).
    floor_shift: both dyadic requantisations as the bare shift Eq. 10 prints."""
    qkv = _arr(qkv, np.int8)
    B, T, Cc, H = dims["B"], dims["T"], dims["C"], dims["H"]
    assert qkv.shape == (B * T, 3 * Cc)
    rel_bias = None if rel_bias is None else _arr(rel_bias, np.int8)
    o = np.empty((B * T, Cc), np.int8)
    sc = np.empty((B, H, T, T), np.int8) if want_taps else None
    pr = np.empty((B, H, T, T), np.int8) if want_taps else None
    mask = None if mask is None else _arr(mask, np.int8)
    args = (_ptr(qkv), _ptr(rel_bias), _ptr(mask), 1 if mask is None else int(mask.shape[0]), _ptr(o),
            _dims(dims), _dy(qk_rq), _sp(softmax), _dy(pv_rq), _ptr(sc), _ptr(pr))
    if floor_shift:
        _L().orc_attention_mode(*args, 1)
    else:
        _L().orc_attention_masked(*args)
    return (o, sc, pr) if want_taps else o


_PTR_FIELDS = {
    "ln1_gamma": np.int32, "ln1_beta": np.int32, "w_qkv": np.int8, "bias_qkv": np.int32, "qkv_rq_b": np.int32,
    "qkv_rq_c": np.int32, "rel_bias": np.int8, "w_proj": np.int8, "bias_proj": np.int32, "proj_rq_b": np.int32,
    "proj_rq_c": np.int32, "ln2_gamma": np.int32, "ln2_beta": np.int32, "w_fc1": np.int8, "bias_fc1": np.int32,
    "fc1_rq_b": np.int32, "fc1_rq_c": np.int32, "w_fc2": np.int8, "bias_fc2": np.int32, "fc2_rq_b": np.int32,
    "fc2_rq_c": np.int32, "attn_mask": np.int8,
}
_INT_FIELDS = ("ln1_f_bits", "ln1_c_shift", "ln2_f_bits", "ln2_c_shift")
_DY_FIELDS = ("qk_rq", "pv_rq", "res1_rq", "gelu_rq", "res2_rq")
_SP_FIELDS = ("softmax", "gelu")


def _block(p, keep):
    """Build the C struct from a dict of numpy arrays / ints / tuples / dicts."""
    bp = _BlockParams()
    for name, dt in _PTR_FIELDS.items():
        a = p.get(name)
        if a is None:
            setattr(bp, name, None)
        else:
            a = _arr(a, dt); keep.append(a)
            setattr(bp, name, a.ctypes.data)
    for name in _INT_FIELDS:
        setattr(bp, name, int(p[name]))
    for name in _DY_FIELDS:
        setattr(bp, name, _dy(p[name]))
    for name in _SP_FIELDS:
        setattr(bp, name, _sp(p[name]))
    m = p.get("attn_mask")
    bp.n_mask = 1 if m is None else int(np.shape(m)[0])
    return bp


TAP_NAMES = ("u", "qkv", "scores", "probs", "o", "xhat", "v", "h")


def encoder_block(x, params, dims, want_taps=False):
    """x: int8 [B*T, C].  Returns y, or (y, taps dict) with every intermediate tensor."""
    x = _arr(x, np.int8)
    B, T, Cc, H, F = (dims[k] for k in "BTCHF")
    R = B * T
    assert x.shape == (R, Cc)
    keep = []
    bp = _block(params, keep)
    y = np.empty_like(x)
    taps = None
    tp = None
    if want_taps:
        taps = {"u": np.empty((R, Cc), np.int8), "qkv": np.empty((R, 3 * Cc), np.int8),
                "scores": np.empty((B, H, T, T), np.int8), "probs": np.empty((B, H, T, T), np.int8),
                "o": np.empty((R, Cc), np.int8), "xhat": np.empty((R, Cc), np.int8),
                "v": np.empty((R, Cc), np.int8), "h": np.empty((R, F), np.int8)}
        t = _Taps(*[taps[n].ctypes.data for n in TAP_NAMES])
        tp = C.pointer(t)
    _L().orc_encoder_block(_ptr(x), _ptr(y), C.byref(bp), _dims(dims), tp)
    return (y, taps) if want_taps else y


def forward(x, blocks, dims, final_ln=None):
    """x: int8 [B*T, C]; blocks: list of parameter dicts; final_ln: None or dict(gamma, beta, f_bits, c_shift)."""
    x = _arr(x, np.int8)
    keep = []
    arr = (_BlockParams * len(blocks))(*[_block(p, keep) for p in blocks])
    y = np.empty_like(x)
    if final_ln is None:
        g = b = None; fb = cs = 0
    else:
        g = _arr(final_ln["gamma"], np.int32); b = _arr(final_ln["beta"], np.int32)
        fb, cs = int(final_ln["f_bits"]), int(final_ln["c_shift"])
    _L().orc_forward(_ptr(x), _ptr(y), arr, len(blocks), _ptr(g), _ptr(b), fb, cs, _dims(dims))
    return y


# ---- host-side conversions (Sec. 3.1 Eq. 6, the dyadic number of Sec. 3.2, I_0 of Algorithm 1), exact rationals
def quantize_symmetric(r, m, k=8):
    """clamp(round(r / S)), S = m / (2^(k-1) - 1), ties away from zero; every float is taken as the exact rational it is."""
    from fractions import Fraction
    import math
    qmax = (1 << (k - 1)) - 1
    S = Fraction(float(np.float32(m))) / qmax
    out = np.empty(np.shape(r), np.int8)
    flat = out.reshape(-1)
    for i, v in enumerate(np.asarray(r, np.float32).reshape(-1)):
        if not math.isfinite(float(v)):
            flat[i] = 0 if math.isnan(float(v)) else (qmax if v > 0 else -qmax)
            continue
        t = Fraction(float(v)) / S
        n = math.floor(abs(t) + Fraction(1, 2))
        flat[i] = max(-qmax, min(qmax, n if t >= 0 else -n))
    return out, float(S)


def dyadic_from_float(x, bits=15):
    """(b, c) with b = round(x 2^c), c = bits - 1 - floor(log2 x) limited to [1, 46]; a carry into bit `bits` lowers c."""
    from fractions import Fraction
    import math
    X = Fraction(float(x))
    fl = math.floor(math.log2(X)) if X > 0 else None
    while Fraction(2) ** fl > X:
        fl -= 1
    while Fraction(2) ** (fl + 1) <= X:
        fl += 1
    c = max(1, min(46, bits - 1 - fl))
    rnd = lambda t: math.floor(t + Fraction(1, 2))
    b = rnd(X * 2 ** c)
    if b >= 2 ** bits and c > 1:
        c -= 1
        b = rnd(X * 2 ** c)
    return max(1, b), c


def shift_params_from_scale(s, width=16, m_bits=31, k_out=8):
    from fractions import Fraction
    import math
    i0 = max(1, math.floor(1 / Fraction(float(s)) + Fraction(1, 2)))
    return dict(i0=i0, n_shift=width - i0.bit_length(), m_bits=m_bits, k_out=k_out)


# ---- embedding layer and classifier head (Sec. 3.1; Sec. 3.2: the embedding Conv follows the dyadic pipeline)
def embed_tokens(patch_tok, cls, pos, tok_rq, pos_rq, B):
    """tokens[b, 0] from the class token, tokens[b, 1 + p] from patch_tok[b, p]; each rescaled by tok_rq, plus the
    position embedding rescaled by pos_rq, clamped to int8 (the two-scale addition of the residuals)."""
    patch_tok = _arr(patch_tok, np.int8); cls = _arr(cls, np.int8); pos = _arr(pos, np.int8)
    T, Cc = pos.shape
    P = T - 1
    src = np.empty((B, T, Cc), np.int64)
    src[:, 0, :] = cls.astype(np.int64)
    src[:, 1:, :] = patch_tok.reshape(B, P, Cc).astype(np.int64)
    bt, ct = tok_rq
    bp, cp = pos_rq
    a = (src * int(bt) + (1 << (int(ct) - 1))) >> int(ct)                      # numpy >> on int64 is arithmetic
    q = (pos.astype(np.int64)[None] * int(bp) + (1 << (int(cp) - 1))) >> int(cp)
    return np.clip(a + q, -127, 127).astype(np.int8).reshape(B * T, Cc)


def classifier_head(tokens, T, w, bias, rq_b, rq_c):
    """Dense + requant on row 0 of every image."""
    tokens = _arr(tokens, np.int8)
    return linear_requant(np.ascontiguousarray(tokens[::T]), w, bias, rq_b, rq_c)


def forward_image(patches, image, blocks, d, final_ln):
    B, T = d["B"], d["T"]
    tok = linear_requant(patches, image["w_patch"], image["bias_patch"], image["patch_rq_b"], image["patch_rq_c"])
    x = embed_tokens(tok, image["cls"], image["pos"], image["tok_rq"], image["pos_rq"], B)
    y = forward(x, blocks, d, final_ln=final_ln)
    return classifier_head(y, T, image["w_head"], image["bias_head"], image["head_rq_b"], image["head_rq_c"])


# ---- windowed models (the Swin rows of Table 1): the integer ops above inside the window / stage structure of
# the Swin Transformer, written with plain numpy reshapes.  Tokens of an image are kept in raster order [B, g, g, C].
def window_partition(x, window):
    """[B, g, g, C] -> [B * (g / window)^2, window^2, C], windows in raster order, tokens of a window in raster order."""
    B, g, _, Cc = x.shape
    n = g // window
    return x.reshape(B, n, window, n, window, Cc).transpose(0, 1, 3, 2, 4, 5).reshape(B * n * n, window * window, Cc)


def window_reverse(xw, window, g):
    """Inverse of window_partition."""
    n = g // window
    Cc = xw.shape[-1]
    B = xw.shape[0] // (n * n)
    return xw.reshape(B, n, n, window, window, Cc).transpose(0, 1, 3, 2, 4, 5).reshape(B, g, g, Cc)


def shift_mask(g, window, shift):
    """int8 [(g / window)^2, window^2, window^2]: 1 where two tokens of a window of the cyclically shifted image come
    from different regions of the image (three bands per axis: untouched windows, the unwrapped and the wrapped part of
    the last window), else 0."""
    label = np.zeros((1, g, g, 1), np.int32)
    bands = (slice(0, g - window), slice(g - window, g - shift), slice(g - shift, g))
    n = 0
    for rows in bands:
        for cols in bands:
            label[0, rows, cols, 0] = n
            n += 1
    lw = window_partition(label, window)[:, :, 0]
    return (lw[:, :, None] != lw[:, None, :]).astype(np.int8)


def swin_block(x, p, g, window, shift, H):
    """One block on x int8 [B, g, g, C]: I-LayerNorm, cyclic shift by -shift, window partition, attention per window
    (relative-position bias, mask when shifted), reverse, shift back, projection + residual, then the MLP half."""
    B, _, _, Cc = x.shape
    F = np.shape(p["w_fc1"])[0]
    flat = x.reshape(-1, Cc)
    u = ilayernorm(flat, p["ln1_gamma"], p["ln1_beta"], p["ln1_f_bits"], p["ln1_c_shift"]).reshape(B, g, g, Cc)
    if shift:
        u = np.roll(u, (-shift, -shift), axis=(1, 2))
    uw = window_partition(u, window)
    nW = uw.shape[0]
    qkv = linear_requant(uw.reshape(-1, Cc), p["w_qkv"], p["bias_qkv"], p["qkv_rq_b"], p["qkv_rq_c"])
    d = dict(B=nW, T=window * window, C=Cc, H=H, F=F)
    o = attention(qkv, d, p["qk_rq"], p["softmax"], p["pv_rq"], rel_bias=p.get("rel_bias"),
                  mask=shift_mask(g, window, shift) if shift else None)
    o = window_reverse(o.reshape(nW, window * window, Cc), window, g)
    if shift:
        o = np.roll(o, (shift, shift), axis=(1, 2))
    xhat = linear_requant(o.reshape(-1, Cc), p["w_proj"], p["bias_proj"], p["proj_rq_b"], p["proj_rq_c"],
                          residual=flat, res_rq=p["res1_rq"])
    v = ilayernorm(xhat, p["ln2_gamma"], p["ln2_beta"], p["ln2_f_bits"], p["ln2_c_shift"])
    h = linear_requant(v, p["w_fc1"], p["bias_fc1"], p["fc1_rq_b"], p["fc1_rq_c"], gelu=p["gelu"], gelu_rq=p["gelu_rq"])
    y = linear_requant(h, p["w_fc2"], p["bias_fc2"], p["fc2_rq_b"], p["fc2_rq_c"], residual=xhat, res_rq=p["res2_rq"])
    return y.reshape(B, g, g, Cc)


def patch_merge(x, m):
    """[B, g, g, C] -> [B, g/2, g/2, 2C]: the four tokens of each 2 x 2 neighbourhood are concatenated in the order
    (row, column) offsets (0,0), (1,0), (0,1), (1,1), normalised by I-LayerNorm over 4C and reduced by a Dense layer
    without bias."""
    B, g, _, Cc = x.shape
    cat = np.concatenate([x[:, 0::2, 0::2], x[:, 1::2, 0::2], x[:, 0::2, 1::2], x[:, 1::2, 1::2]], axis=-1)
    u = ilayernorm(cat.reshape(-1, 4 * Cc), m["ln_gamma"], m["ln_beta"], m["f_bits"], m["c_shift"])
    y = linear_requant(u, m["w"], None, m["rq_b"], m["rq_c"])
    return y.reshape(B, g // 2, g // 2, -1)


def mean_pool(x, rq):
    """Average over the tokens of each image as a dyadic rescale of the token sum (the factor 1 / T sits in b / 2^c):
    x int8 [B, T, C] -> int8 [B, C]."""
    x = _arr(x, np.int8)
    s = x.astype(np.int64).sum(axis=1)
    return requant_vec(s, rq[0], rq[1]).astype(np.int8).reshape(s.shape)


def swin_forward(patches, model, want_stages=False):
    """patches int8 [B * g0 * g0, patch_dim] -> logits int8 [B, n_classes].  model: dict(grid, window, embed, stages,
    final_ln, pool_rq, head); a stage is dict(C, H, merge (None for the first), blocks), a block carries `shift`."""
    g, window = model["grid"], model["window"]
    e = model["embed"]
    B = patches.shape[0] // (g * g)
    tok = linear_requant(patches, e["w"], e["bias"], e["rq_b"], e["rq_c"])
    tok = ilayernorm(tok, e["ln_gamma"], e["ln_beta"], e["f_bits"], e["c_shift"])
    x = tok.reshape(B, g, g, -1)
    outs = []
    for st in model["stages"]:
        if st["merge"] is not None:
            x = patch_merge(x, st["merge"])
            g //= 2
        for p in st["blocks"]:
            x = swin_block(x, p, g, window, p["shift"], st["H"])
        outs.append(x.reshape(B * g * g, -1).copy())
    f = model["final_ln"]
    Cc = x.shape[-1]
    z = ilayernorm(x.reshape(-1, Cc), f["gamma"], f["beta"], f["f_bits"], f["c_shift"])
    pooled = mean_pool(z.reshape(B, g * g, Cc), model["pool_rq"])
    hd = model["head"]
    logits = linear_requant(pooled, hd["w"], hd["bias"], hd["rq_b"], hd["rq_c"])
    return (logits, outs, pooled) if want_stages else logits
