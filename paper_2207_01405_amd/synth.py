"""Seeded synthetic workloads for the integer-only ViT encoder (numpy only).

This module serves both the GPU library's tests/benchmark and the CPU oracle's
tests.  It holds none of the method's arithmetic: it only draws random int8 /
int32 tensors with the shapes and value distributions of the ViT / DeiT / Swin
workloads the paper measures (ImageNet-trained checkpoints are not available, so
these stand in for them), and picks dyadic shift counts from closed-form
estimates of accumulator spread so that tensors neither saturate nor collapse.

A block's parameters are a flat dict: numpy arrays for tensors, ints for shift
counts, (b, c) tuples for per-tensor dyadic pairs and dicts(i0, n_shift, m_bits,
k_out) for the Shiftmax / ShiftGELU parameters.
"""
import math

import numpy as np

# name -> shape of the workload.  B = images (or windows), T tokens, C width, H heads, F MLP width, L blocks.
CONFIGS = {
    "c0_tiny":   dict(B=1,    T=65,  C=64,  H=2,  F=256,  L=1,  seed=0, act="normal",   i0="fixed", rel_bias=False),
    "c1_deit_t": dict(B=64,   T=197, C=192, H=3,  F=768,  L=12, seed=1, act="normal",   i0="fixed", rel_bias=False),
    "c2_deit_s": dict(B=128,  T=197, C=384, H=6,  F=1536, L=12, seed=2, act="normal",   i0="loguniform", rel_bias=False),
    "c3_vit_b":  dict(B=256,  T=197, C=768, H=12, F=3072, L=12, seed=3, act="student_t", i0="fixed", rel_bias=False),
    "c4_swin_t": dict(B=8192, T=49,  C=96,  H=3,  F=384,  L=1,  seed=4, act="normal",   i0="fixed", rel_bias=True),
}

for _name, _cfg in CONFIGS.items():
    _cfg["name"] = _name

K_OUT = 8        # output bit width of Shiftmax / ShiftGELU's IntDiv
ACC_BITS = 16    # "16-bit accumulation width": I_0 << N stays below 2^16
M_BITS = 31      # M of IntDiv
LN_F_BITS = 16   # F of the I-LayerNorm reciprocal
LN_C_SHIFT = 19  # final rounded shift of I-LayerNorm
LN_OUT_SCALE = 1.0 / 32.0


def dims_of(cfg, B=None):
    return dict(B=cfg["B"] if B is None else B, T=cfg["T"], C=cfg["C"], H=cfg["H"], F=cfg["F"])


def shift_params(i0):
    """Shiftmax / ShiftGELU parameters for I_0: N chosen so that I_0 * 2^N < 2^ACC_BITS."""
    return dict(i0=int(i0), n_shift=ACC_BITS - int(i0).bit_length(), m_bits=M_BITS, k_out=K_OUT)


def quantize_act(z):
    """Symmetric int8 quantisation of activations with scale 4/127."""
    return np.clip(np.rint(z * (127.0 / 4.0)), -127, 127).astype(np.int8)


def make_input(cfg, B=None, seed_offset=0):
    """int8 tokens [B*T, C]: N(0,1) or Student-t(3) values quantised with scale 4/127."""
    B = cfg["B"] if B is None else B
    rng = np.random.default_rng([cfg["seed"], 1000 + seed_offset])
    n = (B * cfg["T"], cfg["C"])
    z = rng.standard_t(3.0, size=n) if cfg["act"] == "student_t" else rng.standard_normal(n)
    return quantize_act(z)


def _weights(rng, n_out, k):
    """N(0, 0.02^2) weights, per-output-channel symmetric int8.  Returns (w_q, per-channel scale)."""
    w = rng.standard_normal((n_out, k)) * 0.02
    s = np.abs(w).max(axis=1) / 127.0
    return np.clip(np.rint(w / s[:, None]), -127, 127).astype(np.int8), s


MEAN_B = 1.5 * 2.0 ** 14    # mean of a multiplier drawn uniformly from [2^14, 2^15)


def _shift_for(sigma_acc, sigma_target):
    """Shift count in [20, 24] that brings an accumulator of spread sigma_acc closest to sigma_target
    for a multiplier of mean size; also returns the spread that shift is expected to give."""
    c = round(math.log2(max(sigma_acc, 1.0) * MEAN_B / sigma_target))
    c = int(min(24, max(20, c)))
    return c, sigma_acc * MEAN_B / 2.0 ** c


def _dense(rng, n_out, k, sigma_in, sigma_target, s_in):
    """Weights, int32 bias, per-channel multipliers, one shift count for the layer, expected output spread."""
    w, s = _weights(rng, n_out, k)
    sigma_acc = math.sqrt(k) * sigma_in * float(w.astype(np.float64).std())
    c, sigma_out = _shift_for(sigma_acc, sigma_target)
    bias = np.clip(np.rint(rng.standard_normal(n_out) * 0.02 / (s_in * s)), -2 ** 20, 2 ** 20).astype(np.int32)
    rq_b = rng.integers(2 ** 14, 2 ** 15, size=n_out, dtype=np.int64).astype(np.int32)
    rq_c = np.full(n_out, c, np.int32)
    return (w, bias, rq_b, rq_c), min(sigma_out, 127.0)


def _pair(rng, sigma_acc, sigma_target):
    c, sigma_out = _shift_for(sigma_acc, sigma_target)
    return (int(rng.integers(2 ** 14, 2 ** 15)), c), min(sigma_out, 127.0)


def _ln(rng, C):
    gamma = 1.0 + 0.1 * rng.standard_normal(C)
    beta = 0.1 * rng.standard_normal(C)
    gq = np.rint(gamma * 2.0 ** (LN_C_SHIFT - LN_F_BITS) / LN_OUT_SCALE).astype(np.int32)
    bq = np.rint(beta * 2.0 ** LN_C_SHIFT / LN_OUT_SCALE).astype(np.int32)
    return gq, bq


def make_block(cfg, layer):
    """Parameters of encoder block `layer` of the workload `cfg` (deterministic in (cfg.seed, layer))."""
    rng = np.random.default_rng([cfg["seed"], 2000 + layer])
    T, C, H, F = cfg["T"], cfg["C"], cfg["H"], cfg["F"]
    d = C // H
    if cfg["i0"] == "loguniform":       # per-layer activation scale S, log-uniform in [2^-6, 2^-2]
        S = 2.0 ** rng.uniform(-6.0, -2.0)
        i0 = int(round(1.0 / S))
        sig_t = float(min(40.0, max(8.0, 1.0 / S)))
    else:
        i0 = 32                          # round(127 / 4)
        sig_t = 32.0
    sig_ln = 1.0 / LN_OUT_SCALE          # spread of an I-LayerNorm output
    p = {}
    p["ln1_gamma"], p["ln1_beta"] = _ln(rng, C)
    p["ln1_f_bits"], p["ln1_c_shift"] = LN_F_BITS, LN_C_SHIFT
    (p["w_qkv"], p["bias_qkv"], p["qkv_rq_b"], p["qkv_rq_c"]), sig_qkv = \
        _dense(rng, 3 * C, C, sig_ln, sig_t, LN_OUT_SCALE)
    p["qk_rq"], sig_s = _pair(rng, math.sqrt(d) * sig_qkv * sig_qkv, sig_t)
    p["rel_bias"] = (np.clip(np.rint(rng.standard_normal((H, T, T)) * 8.0), -127, 127).astype(np.int8)
                     if cfg["rel_bias"] else None)
    p["softmax"] = shift_params(i0)
    # spread of sum_j P_j V_j for softmax weights of Gaussian logits of spread s: sigma_v * 128 * sqrt(e^(s^2) / T)
    s_logit = math.hypot(sig_s, 8.0 if cfg["rel_bias"] else 0.0) / i0
    sig_pv = sig_qkv * 128.0 * math.sqrt(min(1.0, math.exp(s_logit ** 2) / T))
    p["pv_rq"], sig_o = _pair(rng, sig_pv, sig_t)
    # the two Dense layers that feed the residual stream aim a little lower so that the stream stays in range
    (p["w_proj"], p["bias_proj"], p["proj_rq_b"], p["proj_rq_c"]), _ = \
        _dense(rng, C, C, sig_o, 0.75 * sig_t, LN_OUT_SCALE)
    p["res1_rq"] = (int(rng.integers(2 ** 14, 2 ** 15)), 15)
    p["ln2_gamma"], p["ln2_beta"] = _ln(rng, C)
    p["ln2_f_bits"], p["ln2_c_shift"] = LN_F_BITS, LN_C_SHIFT
    (p["w_fc1"], p["bias_fc1"], p["fc1_rq_b"], p["fc1_rq_c"]), sig_h = \
        _dense(rng, F, C, sig_ln, sig_t, LN_OUT_SCALE)
    p["gelu"] = shift_params(i0)
    # ShiftGELU's raw output is about I * 2^(k-1) * sigmoid(1.702 S I): spread about 0.65 * 128 * sigma_in
    p["gelu_rq"], sig_g = _pair(rng, 0.65 * 128.0 * sig_h, sig_t)
    (p["w_fc2"], p["bias_fc2"], p["fc2_rq_b"], p["fc2_rq_c"]), _ = \
        _dense(rng, C, F, sig_g, 0.75 * sig_t, LN_OUT_SCALE)
    p["res2_rq"] = (int(rng.integers(2 ** 14, 2 ** 15)), 15)
    return p


def make_shift_mask(window=7, shift=3, grid=8):
    """int8 [grid * grid, window^2, window^2] mask of shifted-window attention for one image: after a cyclic shift by
    `shift`, the last row and column of windows hold tokens of different image regions; pairs from different regions
    are masked (1), all other entries are 0.  Window order is row-major over the image, as the tokens are laid out."""
    T = window * window
    m = np.zeros((grid * grid, T, T), np.int8)
    for wy in range(grid):
        for wx in range(grid):
            region = np.zeros((window, window), np.int32)
            if wy == grid - 1:
                region[window - shift:, :] += 1
            if wx == grid - 1:
                region[:, window - shift:] += 2
            r = region.reshape(-1)
            m[wy * grid + wx] = (r[:, None] != r[None, :]).astype(np.int8)
    return m


def make_final_ln(cfg):
    rng = np.random.default_rng([cfg["seed"], 3000])
    g, b = _ln(rng, cfg["C"])
    return dict(gamma=g, beta=b, f_bits=LN_F_BITS, c_shift=LN_C_SHIFT)


PATCH_DIM = {"c0_tiny": 48, "c1_deit_t": 768, "c2_deit_s": 768, "c3_vit_b": 768}     # 4x4x3 for the tiny case, else 16x16x3
N_CLASSES = {"c0_tiny": 10, "c1_deit_t": 1000, "c2_deit_s": 1000, "c3_vit_b": 1000}


def make_image_params(cfg):
    """Embedding layer (patch Dense, class token, position embedding) and classifier head of the workload `cfg`."""
    rng = np.random.default_rng([cfg["seed"], 6000])
    T, C = cfg["T"], cfg["C"]
    kp, ncls = PATCH_DIM[cfg["name"]], N_CLASSES[cfg["name"]]
    p = {}
    (p["w_patch"], p["bias_patch"], p["patch_rq_b"], p["patch_rq_c"]), _ = _dense(rng, C, kp, 32.0, 32.0, LN_OUT_SCALE)
    p["cls"] = np.clip(np.rint(rng.standard_normal(C) * 32.0), -127, 127).astype(np.int8)
    p["pos"] = np.clip(np.rint(rng.standard_normal((T, C)) * 24.0), -127, 127).astype(np.int8)
    p["tok_rq"] = (int(rng.integers(2 ** 14, 2 ** 15)), 15)
    p["pos_rq"] = (int(rng.integers(2 ** 13, 2 ** 14)), 15)
    (p["w_head"], p["bias_head"], p["head_rq_b"], p["head_rq_c"]), _ = _dense(rng, ncls, C, 1.0 / LN_OUT_SCALE, 32.0, LN_OUT_SCALE)
    return p


def make_patches(cfg, n_images=None):
    """int8 [B * (T - 1), patch_dim]: flattened image patches (cutting an image into patches is a permutation)."""
    rng = np.random.default_rng([cfg["seed"], 7000])
    B = cfg["B"] if n_images is None else n_images
    z = rng.standard_normal((max(B, cfg["B"]) * (cfg["T"] - 1), PATCH_DIM[cfg["name"]])) * 32.0
    return np.clip(np.rint(z), -127, 127).astype(np.int8)[: B * (cfg["T"] - 1)]


# Hierarchical windowed models (the Swin rows of Table 1).  grid = tokens per image side after the patch embedding,
# window = tokens per window side; stage s has width C * 2^s and depths[s] blocks that alternate between plain and
# shifted windows (no shift once a window covers the whole grid).
SWIN = {
    "swin_tiny_test": dict(grid=16, window=4, C=32, heads=(1, 2, 4), depths=(2, 2, 2), patch_dim=48, n_classes=10,
                           B=2, seed=11),
    "swin_t": dict(grid=56, window=7, C=96, heads=(3, 6, 12, 24), depths=(2, 2, 6, 2), patch_dim=48, n_classes=1000,
                   B=128, seed=12),
    "swin_s": dict(grid=56, window=7, C=96, heads=(3, 6, 12, 24), depths=(2, 2, 18, 2), patch_dim=48, n_classes=1000,
                   B=128, seed=13),
}

for _name, _cfg in SWIN.items():
    _cfg["name"] = _name


def make_swin_model(cfg):
    """Every parameter of a windowed model: embedding (patch Dense + I-LayerNorm), per stage the patch merging
    (I-LayerNorm over 4C + Dense to 2C, absent for the first stage) and its blocks (each with `shift` and a
    relative-position bias), final I-LayerNorm, pooling pair and head."""
    rng = np.random.default_rng([cfg["seed"], 8000])
    window, T = cfg["window"], cfg["window"] ** 2
    m = dict(grid=cfg["grid"], window=window, patch_dim=cfg["patch_dim"], n_classes=cfg["n_classes"])
    C = cfg["C"]
    (w, bias, rq_b, rq_c), _ = _dense(rng, C, cfg["patch_dim"], 32.0, 32.0, LN_OUT_SCALE)
    g_, b_ = _ln(rng, C)
    m["embed"] = dict(w=w, bias=bias, rq_b=rq_b, rq_c=rq_c, ln_gamma=g_, ln_beta=b_, f_bits=LN_F_BITS, c_shift=LN_C_SHIFT)
    stages = []
    g = cfg["grid"]
    for s, (H, depth) in enumerate(zip(cfg["heads"], cfg["depths"])):
        merge = None
        if s > 0:
            (w, _b, rq_b, rq_c), _ = _dense(rng, 2 * C, 4 * C, 1.0 / LN_OUT_SCALE, 32.0, LN_OUT_SCALE)
            g_, b_ = _ln(rng, 4 * C)
            merge = dict(ln_gamma=g_, ln_beta=b_, f_bits=LN_F_BITS, c_shift=LN_C_SHIFT, w=w, rq_b=rq_b, rq_c=rq_c)
            C *= 2
            g //= 2
        bcfg = dict(T=T, C=C, H=H, F=4 * C, seed=cfg["seed"], i0="fixed", rel_bias=True)
        blocks = []
        for l in range(depth):
            p = make_block(bcfg, 100 * s + l)
            p["shift"] = window // 2 if (l % 2 == 1 and g > window) else 0
            blocks.append(p)
        stages.append(dict(C=C, H=H, grid=g, merge=merge, blocks=blocks))
    m["stages"] = stages
    g_, b_ = _ln(rng, C)
    m["final_ln"] = dict(gamma=g_, beta=b_, f_bits=LN_F_BITS, c_shift=LN_C_SHIFT)
    # the pooled mean of g * g int8 tokens, brought back to int8 at the same scale: b / 2^c ~ 1 / (g * g)
    c = 20
    m["pool_rq"] = (int(round(2.0 ** c / (g * g))), c)
    (w, bias, rq_b, rq_c), _ = _dense(rng, cfg["n_classes"], C, 32.0, 32.0, LN_OUT_SCALE)
    m["head"] = dict(w=w, bias=bias, rq_b=rq_b, rq_c=rq_c)
    return m


def make_swin_patches(cfg, n_images=None):
    """int8 [B * grid^2, patch_dim]: flattened image patches in raster order."""
    rng = np.random.default_rng([cfg["seed"], 9000])
    B = cfg["B"] if n_images is None else n_images
    z = rng.standard_normal((B * cfg["grid"] ** 2, cfg["patch_dim"])) * 32.0
    return np.clip(np.rint(z), -127, 127).astype(np.int8)


def make_model(cfg, n_blocks=None):
    n_blocks = cfg["L"] if n_blocks is None else n_blocks
    return [make_block(cfg, l) for l in range(n_blocks)]


# ------------------------------------------------------------ op-level inputs
def make_rows(seed, rows, cols, dist="normal", sigma=32.0):
    """int8 [rows, cols] test rows: 'normal' (given sigma), 'student_t' (heavy tails), 'uniform', 'const'."""
    rng = np.random.default_rng([seed, 4000])
    if dist == "normal":
        z = rng.standard_normal((rows, cols)) * sigma
    elif dist == "student_t":
        z = rng.standard_t(3.0, size=(rows, cols)) * sigma
    elif dist == "uniform":
        z = rng.integers(-127, 128, size=(rows, cols)).astype(np.float64)
    elif dist == "const":
        z = np.repeat(rng.integers(-127, 128, size=(rows, 1)), cols, axis=1).astype(np.float64)
    else:
        raise ValueError(dist)
    return np.clip(np.rint(z), -127, 127).astype(np.int8)


def make_linear(seed, N, K, sigma_in=32.0, sigma_target=32.0):
    """Weights, bias and per-channel dyadic pairs of one Dense layer."""
    rng = np.random.default_rng([seed, 5000])
    return _dense(rng, N, K, sigma_in, sigma_target, LN_OUT_SCALE)[0]
