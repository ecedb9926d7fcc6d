"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and rejects
bad arguments with the documented status before anything is launched (so none of this needs a GPU)."""
import ctypes as C
import os
import re

import pytest

from paper_2207_01405_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2207_01405_amd import build
        build.build_lib()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    text = open(os.path.join(ROOT, "include", "ivit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ivit_[a-z0-9_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS), declared ^ set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layouts_match_the_header(lib):
    assert C.sizeof(binding.ShiftParams) == 16 and C.sizeof(binding.Dyadic) == 8 and C.sizeof(binding.Dims) == 20
    assert C.sizeof(binding.DebugTaps) == 64 and C.sizeof(binding.FinalLN) == 24
    # pointers 8-byte aligned, ints packed in pairs: count by hand from the header
    n_ptr = sum(1 for _, t in binding.BlockParams._fields_ if t is C.c_void_p)
    # 22 pointers, 4 I-LayerNorm ints, 5 dyadic pairs, 2 shift-parameter structs, n_mask padded to 8 bytes
    assert n_ptr == 22 and C.sizeof(binding.BlockParams) == 22 * 8 + 4 * 4 + 5 * 8 + 2 * 16 + 8
    assert C.sizeof(binding.ImageParams) == 10 * 8 + 2 * 8 + 2 * 8        # 10 pointers, 2 ints each padded, 2 dyadic pairs


def test_strerror(lib):
    assert binding.strerror(0) == "ok"
    for code in binding.ERRORS.values():
        assert binding.strerror(code) not in ("ok", "unknown status")
    assert binding.strerror(-99) == "unknown status"


FAKE = 0x10000          # a non-NULL, 16-byte aligned address that is never dereferenced: validation fails first
SP = binding.ShiftParams(32, 10, 31, 8)
DY = binding.Dyadic(20000, 20)
E = binding.ERRORS


def _lin(lib, x=FAKE, w=FAKE, bias=None, b=FAKE, c=FAKE, res=None, res_rq=DY, gelu=None, gelu_rq=DY, y=FAKE, M=8, N=8, K=16):
    g = None if gelu is None else C.byref(gelu)
    return lib.ivit_linear_requant(None, x, w, bias, b, c, res, res_rq, g, gelu_rq, y, M, N, K)


def test_linear_rejects_bad_arguments(lib):
    assert _lin(lib, x=None) == E["NULL"] and _lin(lib, y=None) == E["NULL"] and _lin(lib, b=None) == E["NULL"]
    assert _lin(lib, M=-1) == E["SHAPE"] and _lin(lib, N=0) == E["SHAPE"]
    assert _lin(lib, K=0) == E["SHAPE"] and _lin(lib, K=24) == E["SHAPE"] and _lin(lib, K=65552) == E["SHAPE"]
    assert _lin(lib, x=FAKE + 4) == E["ALIGN"] and _lin(lib, b=FAKE + 2) == E["ALIGN"]
    assert _lin(lib, res=FAKE, res_rq=binding.Dyadic(0, 5)) == E["PARAM"]
    assert _lin(lib, res=FAKE, res_rq=binding.Dyadic(5, 47)) == E["PARAM"]
    assert _lin(lib, res=FAKE, gelu=SP) == E["PARAM"]
    assert _lin(lib, gelu=binding.ShiftParams(0, 10, 31, 8)) == E["PARAM"]
    assert _lin(lib, gelu=binding.ShiftParams(64, 10, 31, 8)) == E["PARAM"]       # 64 << 10 = 65536 > 65535
    assert _lin(lib, gelu=binding.ShiftParams(32, 10, 32, 8)) == E["PARAM"]
    assert _lin(lib, gelu=binding.ShiftParams(32, 10, 31, 9)) == E["PARAM"]
    assert _lin(lib, gelu=SP, gelu_rq=binding.Dyadic(-1, 3)) == E["PARAM"]
    assert _lin(lib, M=0) == 0                                                      # empty input: nothing to do


def test_rowwise_reject_bad_arguments(lib):
    sm = lib.ivit_shiftmax
    assert sm(None, None, None, 1, 1, FAKE, 4, 8, 8, SP) == E["NULL"]
    assert sm(None, FAKE, None, 1, 1, FAKE, -1, 8, 8, SP) == E["SHAPE"]
    assert sm(None, FAKE, None, 1, 1, FAKE, 4, 0, 8, SP) == E["SHAPE"]
    assert sm(None, FAKE, None, 1, 1, FAKE, 4, 1025, 1025, SP) == E["SHAPE"]
    assert sm(None, FAKE, None, 1, 1, FAKE, 4, 8, 7, SP) == E["SHAPE"]
    assert sm(None, FAKE, FAKE, 0, 4, FAKE, 4, 8, 8, SP) == E["SHAPE"]
    assert sm(None, FAKE, None, 1, 1, FAKE, 4, 8, 8, binding.ShiftParams(32, 10, 5, 8)) == E["PARAM"]
    assert sm(None, FAKE, None, 1, 1, FAKE, 0, 8, 8, SP) == 0
    ge = lib.ivit_shiftgelu
    assert ge(None, None, FAKE, 4, SP, DY) == E["NULL"] and ge(None, FAKE, FAKE, -4, SP, DY) == E["SHAPE"]
    assert ge(None, FAKE, FAKE, 4, SP, binding.Dyadic(1, 0)) == E["PARAM"] and ge(None, FAKE, FAKE, 0, SP, DY) == 0
    assert lib.ivit_shiftgelu_raw(None, FAKE, FAKE + 1, 4, SP) == E["ALIGN"]
    ln = lib.ivit_ilayernorm
    assert ln(None, FAKE, None, FAKE, FAKE, 4, 64, 16, 19) == E["NULL"]
    assert ln(None, FAKE, FAKE, FAKE, FAKE, 4, 66, 16, 19) == E["SHAPE"]
    assert ln(None, FAKE, FAKE, FAKE, FAKE, 4, 2048, 16, 19) == E["SHAPE"]
    assert ln(None, FAKE, FAKE, FAKE, FAKE, -4, 64, 16, 19) == E["SHAPE"]
    assert ln(None, FAKE, FAKE, FAKE, FAKE, 4, 64, 21, 19) == E["PARAM"]
    assert ln(None, FAKE, FAKE, FAKE, FAKE, 4, 64, 16, 0) == E["PARAM"]
    assert ln(None, FAKE + 2, FAKE, FAKE, FAKE, 4, 64, 16, 19) == E["ALIGN"]
    assert ln(None, FAKE, FAKE, FAKE, FAKE, 0, 64, 16, 19) == 0


def _fake_block():
    bp = binding.BlockParams()
    for name, t in binding.BlockParams._fields_:
        if t is C.c_void_p:
            setattr(bp, name, FAKE)
    bp.rel_bias = None
    bp.attn_mask = None
    for k in ("ln1_f_bits", "ln2_f_bits"):
        setattr(bp, k, 16)
    for k in ("ln1_c_shift", "ln2_c_shift"):
        setattr(bp, k, 19)
    for k in ("qk_rq", "pv_rq", "res1_rq", "gelu_rq", "res2_rq"):
        setattr(bp, k, DY)
    bp.softmax = SP
    bp.gelu = SP
    return bp


def test_workspace_and_block_validation(lib):
    good = binding.Dims(2, 65, 64, 2, 256)
    nbytes = lib.ivit_workspace_bytes(C.byref(good))
    R = 2 * 65
    # two ping-pong activations, u, o, xhat [R,C] each; qkv [R,3C]; h [R,F]
    assert nbytes >= R * (64 * 5 + 64 * 3 + 256) and nbytes % 256 == 0
    for bad in (binding.Dims(2, 0, 64, 2, 256), binding.Dims(2, 257, 64, 2, 256), binding.Dims(2, 65, 64, 4, 256),
                binding.Dims(2, 65, 60, 2, 256), binding.Dims(-1, 65, 64, 2, 256), binding.Dims(2, 65, 64, 2, 250),
                binding.Dims(2, 65, 2048, 32, 256)):
        assert lib.ivit_workspace_bytes(C.byref(bad)) == 0
        assert lib.ivit_encoder_block(None, FAKE, FAKE, C.byref(_fake_block()), C.byref(bad), FAKE, 1 << 30, None) == E["SHAPE"]
    bp = _fake_block()
    blk = lambda **kw: lib.ivit_encoder_block(None, kw.get("x", FAKE), FAKE, C.byref(kw.get("bp", bp)), C.byref(good),
                                              kw.get("ws", 0x100000), kw.get("n", nbytes), None)
    assert blk(x=None) == E["NULL"]
    assert blk(ws=None) == E["WORKSPACE"] and blk(n=nbytes - 1) == E["WORKSPACE"]
    assert blk(ws=0x100000 + 16) == E["ALIGN"]
    b2 = _fake_block(); b2.w_fc1 = None
    assert blk(bp=b2) == E["NULL"]
    b3 = _fake_block(); b3.softmax = binding.ShiftParams(32, 12, 31, 8)
    assert blk(bp=b3) == E["PARAM"]
    b4 = _fake_block(); b4.res2_rq = binding.Dyadic(0, 1)
    assert blk(bp=b4) == E["PARAM"]
    b5 = _fake_block(); b5.fc2_rq_c = FAKE + 2
    assert blk(bp=b5) == E["ALIGN"]
    # forward: same checks for every block, plus the final LayerNorm
    arr = (binding.BlockParams * 2)(_fake_block(), b3)
    fwd = lambda n, fl=None: lib.ivit_forward(None, FAKE, FAKE, arr, n, fl, C.byref(good), 0x100000, nbytes)
    assert fwd(2) == E["PARAM"] and fwd(-1) == E["SHAPE"]
    assert fwd(1, C.byref(binding.FinalLN(None, FAKE, 16, 19))) == E["NULL"]
    assert fwd(1, C.byref(binding.FinalLN(FAKE, FAKE, 30, 19))) == E["PARAM"]
    att = lambda d, qk=DY: lib.ivit_attention(None, FAKE, None, FAKE, C.byref(d), qk, SP, DY, None, None)
    assert att(binding.Dims(2, 300, 64, 2, 256)) == E["SHAPE"] and att(good, binding.Dyadic(1, 60)) == E["PARAM"]
    empty = binding.Dims(0, 65, 64, 2, 256)
    assert att(empty) == 0 and lib.ivit_workspace_bytes(C.byref(empty)) > 0


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "does_not_exist.so"))
    with pytest.raises(RuntimeError, match="not built"):
        binding.load()


def test_synthetic_configs_fit_the_supported_shapes(lib):
    for cfg in synth.CONFIGS.values():
        d = binding.dims(synth.dims_of(cfg))
        assert lib.ivit_workspace_bytes(C.byref(d)) > 0
