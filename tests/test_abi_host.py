"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and rejects
bad arguments with the documented status before anything is launched (so none of this needs a GPU)."""
import ctypes as C
import os
import re
import subprocess

import numpy as np

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
    # 23 pointers, 4 I-LayerNorm ints, 5 dyadic pairs, 2 shift-parameter structs, n_mask and n_win each padded to 8 bytes
    assert n_ptr == 23 and C.sizeof(binding.BlockParams) == 23 * 8 + 4 * 4 + 5 * 8 + 2 * 16 + 2 * 8
    assert C.sizeof(binding.ImageParams) == 10 * 8 + 2 * 8 + 2 * 8        # 10 pointers, 2 ints each padded, 2 dyadic pairs


def test_struct_sizes_and_offsets_agree_with_a_c_compiler(tmp_path):
    """The header compiled by gcc reports the size of every struct and the offset of every field; ctypes must agree."""
    structs = {"ivit_shift_params": binding.ShiftParams, "ivit_dyadic": binding.Dyadic, "ivit_dims": binding.Dims,
               "ivit_block_params": binding.BlockParams, "ivit_debug_taps": binding.DebugTaps,
               "ivit_final_ln": binding.FinalLN, "ivit_image_params": binding.ImageParams,
               "ivit_swin_stage": binding.SwinStage, "ivit_swin_params": binding.SwinParams}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "ivit.h"', 'int main(void) {']
    for cname, cls in structs.items():
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (cname, cname))
        for fname, _ in cls._fields_:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (cname, fname, cname, fname))
    lines.append("return 0; }")
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for cname, cls in structs.items():
        assert int(out[cname]) == C.sizeof(cls), cname
        for fname, _ in cls._fields_:
            assert int(out["%s.%s" % (cname, fname)]) == getattr(cls, fname).offset, (cname, fname)


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
    rm = lib.ivit_shiftgelu_rowmax
    wide = binding.ShiftParams(32, 24, 46, 8)
    assert rm(None, None, FAKE, 4, 64, wide, DY) == E["NULL"] and rm(None, FAKE, FAKE, -1, 64, wide, DY) == E["SHAPE"]
    assert rm(None, FAKE, FAKE, 4, 66, wide, DY) == E["SHAPE"] and rm(None, FAKE, FAKE, 4, 4100, wide, DY) == E["SHAPE"]
    assert rm(None, FAKE, FAKE, 4, 64, binding.ShiftParams(32, 26, 46, 8), DY) == E["PARAM"]      # 32 << 26 > 2^30
    assert rm(None, FAKE, FAKE, 4, 64, binding.ShiftParams(32, 24, 47, 8), DY) == E["PARAM"]
    assert rm(None, FAKE + 1, FAKE, 4, 64, wide, DY) == E["ALIGN"] and rm(None, None, None, 0, 64, wide, DY) == 0
    ln = lib.ivit_ilayernorm
    assert ln(None, FAKE, None, FAKE, FAKE, 4, 64, 16, 19) == E["NULL"]
    assert ln(None, FAKE, FAKE, FAKE, FAKE, 4, 66, 16, 19) == E["SHAPE"]
    assert ln(None, FAKE, FAKE, FAKE, FAKE, 4, 2052, 16, 19) == E["SHAPE"]
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
    bp.tok_index = None
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


def test_forward_image_checks_everything_before_the_first_launch(lib):
    """A bad block, final LayerNorm, workspace or alignment is reported with its own status.  No GPU is present in the
    host suite, so a call that reached a launch would come back as IVIT_ERR_HIP instead: the status proves that
    nothing was enqueued before the argument was found."""
    good = binding.Dims(2, 65, 64, 2, 256)
    need = lib.ivit_image_workspace_bytes(C.byref(good))
    assert need > lib.ivit_workspace_bytes(C.byref(good))

    def image(**kw):
        ip = binding.ImageParams()
        for name, t in binding.ImageParams._fields_:
            if t is C.c_void_p:
                setattr(ip, name, FAKE)
        ip.patch_dim, ip.n_classes, ip.tok_rq, ip.pos_rq = 48, 10, DY, DY
        for k, v in kw.items():
            setattr(ip, k, v)
        return ip

    fl = binding.FinalLN(FAKE, FAKE, 16, 19)

    def call(ip=None, blocks=None, n=2, fln=fl, ws=0x100000, nbytes=need, dims=good, patches=FAKE):
        arr = blocks if blocks is not None else (binding.BlockParams * 2)(_fake_block(), _fake_block())
        return lib.ivit_forward_image(None, patches, FAKE, C.byref(ip or image()), arr, n, C.byref(fln), C.byref(dims), ws, nbytes)

    bad_block = _fake_block(); bad_block.res2_rq = binding.Dyadic(0, 1)
    assert call(blocks=(binding.BlockParams * 2)(_fake_block(), bad_block)) == E["PARAM"]        # the LAST block is bad
    null_block = _fake_block(); null_block.w_fc2 = None
    assert call(blocks=(binding.BlockParams * 2)(null_block, _fake_block())) == E["NULL"]
    odd_block = _fake_block(); odd_block.qkv_rq_b = FAKE + 2
    assert call(blocks=(binding.BlockParams * 2)(_fake_block(), odd_block)) == E["ALIGN"]
    assert call(fln=binding.FinalLN(FAKE, None, 16, 19)) == E["NULL"]
    assert call(fln=binding.FinalLN(FAKE, FAKE, 21, 19)) == E["PARAM"]
    assert call(ws=None) == E["WORKSPACE"] and call(nbytes=need - 1) == E["WORKSPACE"]
    assert call(ws=0x100000 + 64) == E["ALIGN"] and call(patches=FAKE + 8) == E["ALIGN"]
    assert call(ip=image(cls=None)) == E["NULL"] and call(ip=image(w_head=None)) == E["NULL"]
    assert call(ip=image(pos=FAKE + 4)) == E["ALIGN"] and call(ip=image(head_rq_c=FAKE + 2)) == E["ALIGN"]
    assert call(ip=image(patch_dim=40)) == E["SHAPE"] and call(ip=image(n_classes=0)) == E["SHAPE"]
    assert call(ip=image(tok_rq=binding.Dyadic(0, 3))) == E["PARAM"]
    assert call(n=-1) == E["SHAPE"] and call(dims=binding.Dims(2, 65, 60, 2, 256)) == E["SHAPE"]


def test_linear_options_and_probe_arguments(lib):
    ex = lambda opt, **kw: lib.ivit_linear_requant_ex(None, FAKE, FAKE, None, FAKE, FAKE, kw.get("res"), DY, None, DY, FAKE,
                                                      kw.get("M", 8), kw.get("N", 64), kw.get("K", 384),
                                                      None if opt is None else C.byref(binding.LinearOptions(opt)))
    assert ex(4) == E["PARAM"] and ex(-1) == E["PARAM"]
    # the big-tile kernel takes K % 128 == 0, K >= 384, N % 128 == 0
    assert ex(3, K=384, N=64) == E["SHAPE"] and ex(3, K=256, N=128) == E["SHAPE"] and ex(3, K=448, N=128) == E["SHAPE"]
    assert ex(3, K=384, N=128, M=0) == 0
    bad_round = binding.LinearOptions(0, 2)
    assert lib.ivit_linear_requant_ex(None, FAKE, FAKE, None, FAKE, FAKE, None, DY, None, DY, FAKE, 8, 64, 384, C.byref(bad_round)) == E["PARAM"]
    good = binding.Dims(2, 65, 64, 2, 256)
    wa = lambda opt: lib.ivit_window_attention_ex(None, FAKE, None, None, 1, None, 1, FAKE, C.byref(good), DY, SP, DY, None, None, opt)
    assert wa(C.byref(binding.AttentionOptions(2))) == E["PARAM"] and wa(C.byref(binding.AttentionOptions(-1))) == E["PARAM"]
    empty = binding.Dims(0, 65, 64, 2, 256)
    assert lib.ivit_window_attention_ex(None, None, None, None, 1, None, 1, None, C.byref(empty), DY, SP, DY, None, None,
                                        C.byref(binding.AttentionOptions(1))) == 0
    # the register-stationary kernels take K = 384, 768 or 1536 (192 without a residual) with N % 32 == 0 and nothing else
    assert ex(2, K=192, res=FAKE) == E["SHAPE"] and ex(2, K=192, M=0) == 0
    assert ex(2, K=512) == E["SHAPE"] and ex(2, N=48) == E["SHAPE"] and ex(2, K=3072) == E["SHAPE"]
    assert ex(2, K=1536, N=48) == E["SHAPE"] and ex(2, K=1536, M=0) == 0
    assert ex(2, M=0) == 0 and ex(0, M=0) == 0 and ex(None, M=0) == 0 and ex(1, M=0, K=512) == 0
    ops = C.c_int64(0)
    pr = lambda rnd=0, it=100, s=0x100000, n=1 << 20, o=ops: lib.ivit_probe_mfma_rate(None, rnd, it, s, n, C.byref(o) if o is not None else None)
    assert pr(it=0) == E["PARAM"] and pr(it=(1 << 24) + 1) == E["PARAM"]
    assert pr(s=None) == E["NULL"] and pr(o=None) == E["NULL"]
    assert pr(s=0x100000 + 16) == E["ALIGN"]


def _ln_extreme(Cn, f_bits):
    """Largest |x - mean| * f the definition of Eq. 19-20 gives over rows built to maximise it (brute force)."""
    from oracle import oracle as orc
    best = 0
    rows = []
    for k in range(1, 6):                       # k spikes of height h over a constant floor
        for h in range(1, 256):
            for base in (0, -128, 100):
                r = np.full(Cn, base, np.int64)
                r[:k] = np.clip(base + h, -128, 127) if base <= 0 else base - h
                rows.append(r)
    x = np.stack(rows)
    s = x.sum(1)
    mean = (s + Cn // 2) // Cn
    dev = x - mean[:, None]
    var = (dev * dev).sum(1) // Cn
    std = np.maximum(1, orc.isqrt10_vec(var))
    f = (1 << f_bits) // std
    return int((np.abs(dev).max(1) * f).max())


@pytest.mark.parametrize("Cn", [4, 64, 96, 384, 768, 2048])
def test_ilayernorm_limits_cover_every_row(lib, Cn):
    """The bound behind ivit_ilayernorm_limits, |x - mean| f <= 2 sqrt(C) 2^F, checked by brute force over the rows
    that come closest to it, and the limits themselves: with them the largest value the kernel forms fits 32 bits."""
    for f_bits, c_shift in ((16, 19), (20, 23), (8, 12), (1, 1), (20, 31)):
        g, b = binding.ivit_ilayernorm_limits(Cn, f_bits, c_shift)
        worst = _ln_extreme(Cn, f_bits)
        bound = int(np.ceil(np.sqrt(4 * Cn))) << f_bits
        assert worst <= bound, (worst, bound)
        if f_bits >= 8:
            assert worst > bound // 2, (worst, bound)                       # and not a slack one
        assert b == min(1 << 30, 2 ** 31 - 1 - (1 << (c_shift - 1))) and 0 <= g <= 32767
        assert bound * g + b + (1 << (c_shift - 1)) <= 2 ** 31 - 1
        if g < 32767:
            assert bound * (g + 1) + b + (1 << (c_shift - 1)) > 2 ** 31 - 1
    gm, bm = C.c_int32(), C.c_int32()
    assert lib.ivit_ilayernorm_limits(66, 16, 19, C.byref(gm), C.byref(bm)) == E["SHAPE"]
    assert lib.ivit_ilayernorm_limits(64, 21, 19, C.byref(gm), C.byref(bm)) == E["PARAM"]
    assert lib.ivit_ilayernorm_limits(64, 16, 19, None, C.byref(bm)) == E["NULL"]


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "does_not_exist.so"))
    with pytest.raises(RuntimeError, match="not built"):
        binding.load()


def test_synthetic_configs_fit_the_supported_shapes(lib):
    for cfg in synth.CONFIGS.values():
        d = binding.dims(synth.dims_of(cfg))
        assert lib.ivit_workspace_bytes(C.byref(d)) > 0


# ------------------------------------------------------------------ windowed models: tables, gather, pooling, forward
@pytest.mark.parametrize("g,w,s", [(8, 4, 2), (8, 4, 0), (56, 7, 3), (28, 7, 3), (14, 7, 3), (7, 7, 0), (12, 3, 1), (16, 4, 3)])
def test_window_index_and_shift_mask_match_the_oracle(lib, g, w, s):
    import oracle as orc
    idx = binding.ivit_swin_window_index(g, w, s)
    ids = np.arange(g * g, dtype=np.int32).reshape(1, g, g, 1)
    assert np.array_equal(idx, orc.window_partition(np.roll(ids, (-s, -s), axis=(1, 2)), w)[:, :, 0])
    assert sorted(idx.reshape(-1).tolist()) == list(range(g * g))
    m = binding.ivit_swin_shift_mask(g, w, s)
    assert np.array_equal(m, orc.shift_mask(g, w, s) if s else np.zeros_like(m))


def test_window_tables_reject_bad_arguments(lib):
    buf = (C.c_int32 * 64)()
    assert lib.ivit_swin_window_index(8, 3, 0, buf) == E["SHAPE"] and lib.ivit_swin_window_index(0, 4, 0, buf) == E["SHAPE"]
    assert lib.ivit_swin_window_index(8, 4, 4, buf) == E["PARAM"] and lib.ivit_swin_window_index(8, 4, -1, buf) == E["PARAM"]
    assert lib.ivit_swin_window_index(8, 4, 1, None) == E["NULL"] and lib.ivit_swin_shift_mask(8, 4, 1, None) == E["NULL"]
    assert lib.ivit_swin_shift_mask(8, 5, 1, buf) == E["SHAPE"] and lib.ivit_swin_shift_mask(8, 4, 7, buf) == E["PARAM"]


def test_window_attention_and_small_ops_reject_bad_arguments(lib):
    d = binding.Dims(8, 16, 64, 2, 256)
    wa = lambda rb=FAKE, ti=FAKE, n_win=4, dd=d: lib.ivit_window_attention(None, FAKE, rb, None, 1, ti, n_win, FAKE, C.byref(dd),
                                                                          DY, SP, DY, None, None)
    assert wa(rb=None) == E["NULL"]                      # a table needs the bias
    assert wa(n_win=3) == E["SHAPE"] and wa(n_win=0) == E["SHAPE"]
    assert wa(ti=FAKE + 2) == E["ALIGN"]
    assert wa(dd=binding.Dims(0, 16, 64, 2, 256)) == 0
    pm = lib.ivit_patch_merge_gather
    assert pm(None, FAKE, FAKE, 2, 7, 64) == E["SHAPE"] and pm(None, FAKE, FAKE, 2, 8, 24) == E["SHAPE"]
    assert pm(None, None, FAKE, 2, 8, 64) == E["NULL"] and pm(None, FAKE + 8, FAKE, 2, 8, 64) == E["ALIGN"]
    assert pm(None, None, None, 0, 8, 64) == 0
    mp = lib.ivit_mean_pool
    assert mp(None, FAKE, FAKE, 2, 0, 64, DY) == E["SHAPE"] and mp(None, FAKE, FAKE, 2, 49, 62, DY) == E["SHAPE"]
    assert mp(None, FAKE, None, 2, 49, 64, DY) == E["NULL"] and mp(None, FAKE, FAKE, 2, 49, 64, binding.Dyadic(0, 3)) == E["PARAM"]
    assert mp(None, None, None, 0, 49, 64, DY) == 0


def _fake_swin(grid=16, window=4, C0=32, heads=(1, 2, 4), depths=(2, 2, 2)):
    sp = binding.SwinParams()
    keep = []
    sp.grid, sp.window, sp.n_stages, sp.patch_dim, sp.n_classes = grid, window, len(heads), 48, 10
    for k in ("w_patch", "bias_patch", "patch_rq_b", "patch_rq_c", "w_head", "bias_head", "head_rq_b", "head_rq_c"):
        setattr(sp, k, FAKE)
    ln = binding.FinalLN(FAKE, FAKE, 16, 19)
    sp.embed_ln = ln; sp.final_ln = ln; sp.pool_rq = DY
    g = grid
    for s, (H, n) in enumerate(zip(heads, depths)):
        if s:
            g //= 2
        st = sp.stages[s]
        st.C, st.H, st.F, st.n_blocks = C0 << s, H, 4 * (C0 << s), n
        arr = (binding.BlockParams * n)()
        for l in range(n):
            bp = _fake_block()
            bp.rel_bias = FAKE
            if g > window:
                bp.tok_index = FAKE; bp.n_win = (g // window) ** 2
                if l % 2:
                    bp.attn_mask = FAKE; bp.n_mask = bp.n_win
            arr[l] = bp
        keep.append(arr)
        st.blocks = arr
        if s:
            st.merge_ln = ln; st.w_merge = FAKE; st.merge_rq_b = FAKE; st.merge_rq_c = FAKE
    return sp, keep


def test_forward_swin_validation(lib):
    sp, keep = _fake_swin()
    n = lib.ivit_swin_workspace_bytes(C.byref(sp), 2)
    # four activation-size buffers of the first stage plus the block workspace of the largest stage
    assert n >= 4 * 2 * 256 * 32 + lib.ivit_workspace_bytes(C.byref(binding.Dims(2 * 16, 16, 32, 1, 128))) and n % 256 == 0
    run = lambda p=sp, B=2, ws=0x100000, nb=n, x=FAKE: lib.ivit_forward_swin(None, x, FAKE, C.byref(p), B, ws, nb)
    assert run(ws=None) == E["WORKSPACE"] and run(nb=n - 1) == E["WORKSPACE"] and run(ws=0x100000 + 64) == E["ALIGN"]
    assert run(x=None) == E["NULL"] and run(B=-1) == E["SHAPE"] and run(B=0) == 0
    bad, k2 = _fake_swin(); bad.stages[1].C = 96
    assert run(bad) == E["SHAPE"] and lib.ivit_swin_workspace_bytes(C.byref(bad), 2) == 0
    bad, k2 = _fake_swin(grid=12)                       # 12 -> 6: the windows of 4 do not divide the second stage
    assert run(bad) == E["SHAPE"]
    bad, k2 = _fake_swin(); k2[0][1].tok_index = None   # a multi-window stage needs its table
    assert run(bad) == E["NULL"]
    bad, k2 = _fake_swin(); k2[1][1].n_mask = 3         # mask count differs from the stage's window count
    assert run(bad) == E["SHAPE"]
    bad, k2 = _fake_swin(); k2[0][0].n_win = 4
    assert run(bad) == E["SHAPE"]
    bad, k2 = _fake_swin(); bad.stages[2].w_merge = None
    assert run(bad) == E["NULL"]
    bad, k2 = _fake_swin(); bad.pool_rq = binding.Dyadic(1, 0)
    assert run(bad) == E["PARAM"]
    bad, k2 = _fake_swin(); bad.n_stages = 5
    assert run(bad) == E["SHAPE"]
    bad, k2 = _fake_swin(); k2[2][0].gelu = binding.ShiftParams(0, 1, 31, 8)
    assert run(bad) == E["PARAM"]
    for cfg in synth.SWIN.values():                     # the synthetic windowed models fit
        sp2, k3 = _fake_swin(cfg["grid"], cfg["window"], cfg["C"], cfg["heads"], cfg["depths"])
        assert lib.ivit_swin_workspace_bytes(C.byref(sp2), cfg["B"]) > 0


def test_library_was_built_from_the_present_sources():
    """The build script stamps the library with a digest of its sources; the binding refuses a stale library.  A
    library that does not match means a rebuild was forgotten or failed."""
    from paper_2207_01405_amd import build
    lib = binding.load()
    assert lib.ivit_build_id().decode() == build.source_id()
