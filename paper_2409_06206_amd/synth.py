"""Seeded synthetic inputs for one GSWA layer.

Holds none of the layer's arithmetic: only random draws, shapes and the
host-side rounding of inputs to the storage type.  Both the HIP path and the
CPU oracle are fed from here so that they see identical values.

Shapes follow SwinIR-style image-restoration settings: C in {60, 180}, 6 heads,
8x8 windows, 64x64 training patches; the "agile" cases take the narrow query/key
projections and 12x12 windows of Sec. "Parameter Allocation" on 48x48 patches.
Two value regimes:

* ``init``   x, dy ~ N(0,1); weights and bias table ~ N(0, 0.02^2); linear biases 0
             (the initialisation the Swin family trains from);
* ``stress`` weights ~ N(0, 1/fan_in), bias table ~ N(0,1), linear biases ~ N(0, 0.1^2):
             scores of order 1-5 and peaked softmax rows, so that mask, bias and
             exponent mistakes are visible (the ``init`` regime gives almost uniform rows).
"""
import numpy as np


def param_shapes(C, heads, groups, window, dqk=0):
    """dqk: channels of q and of k per head (0: C // heads); a group projects to
    2 * heads_per_group * dqk + Cg features [q | k | v]."""
    Cg = C // groups
    Rg = 2 * (heads // groups) * (dqk or C // heads) + Cg
    return {
        "w_qkv": (groups, Rg, Cg),
        "b_qkv": (groups, Rg),
        "w_proj": (C, C),
        "b_proj": (C,),
        "table": ((2 * window - 1) ** 2, heads),
    }


def layer_params(C, heads, groups, window, seed, regime="init", dqk=0):
    """fp32 parameters of one layer, drawn in the order w_qkv, w_proj, table, b_qkv, b_proj."""
    rng = np.random.default_rng(seed)
    shp = param_shapes(C, heads, groups, window, dqk)
    Cg = C // groups
    if regime == "init":
        p = {
            "w_qkv": rng.normal(0.0, 0.02, shp["w_qkv"]),
            "w_proj": rng.normal(0.0, 0.02, shp["w_proj"]),
            "table": rng.normal(0.0, 0.02, shp["table"]),
            "b_qkv": np.zeros(shp["b_qkv"]),
            "b_proj": np.zeros(shp["b_proj"]),
        }
    elif regime == "stress":
        p = {
            "w_qkv": rng.normal(0.0, Cg ** -0.5, shp["w_qkv"]),
            "w_proj": rng.normal(0.0, C ** -0.5, shp["w_proj"]),
            "table": rng.normal(0.0, 1.0, shp["table"]),
            "b_qkv": rng.normal(0.0, 0.1, shp["b_qkv"]),
            "b_proj": rng.normal(0.0, 0.1, shp["b_proj"]),
        }
    else:
        raise ValueError(f"unknown regime {regime!r}")
    return {k: v.astype(np.float32) for k, v in p.items()}


def astl_param_shapes(C, heads, groups, window, hidden, dqk=0):
    """Parameters of a whole layer (Eq. 4-5): two LayerNorms, the attention layer's five tensors and
    the two fully connected layers of the MLP (``hidden`` features in between)."""
    shp = {"ln1_w": (C,), "ln1_b": (C,)}
    shp.update(param_shapes(C, heads, groups, window, dqk))
    shp.update({"ln2_w": (C,), "ln2_b": (C,), "w_fc1": (hidden, C), "b_fc1": (hidden,),
                "w_fc2": (C, hidden), "b_fc2": (C,)})
    return shp


def astl_params(C, heads, groups, window, hidden, seed, regime="init", dqk=0):
    """fp32 parameters of a whole layer: the attention tensors as ``layer_params`` draws them from
    ``seed``; then, from ``seed + 5000``, in the order w_fc1, w_fc2, b_fc1, b_fc2, ln1_w, ln1_b,
    ln2_w, ln2_b: ``init`` has fc weights ~ N(0, 0.02^2), zero fc biases and identity LayerNorms
    (gamma 1, beta 0); ``stress`` has fc weights ~ N(0, 1/fan_in), fc biases ~ N(0, 0.1^2),
    gamma ~ 1 + N(0, 0.1^2), beta ~ N(0, 0.1^2), so that both branches are of the order of the
    skip path and every parameter's gradient is visible."""
    p = dict(layer_params(C, heads, groups, window, seed, regime, dqk))
    rng = np.random.default_rng(seed + 5000)
    if regime == "init":
        q = {
            "w_fc1": rng.normal(0.0, 0.02, (hidden, C)),
            "w_fc2": rng.normal(0.0, 0.02, (C, hidden)),
            "b_fc1": np.zeros(hidden), "b_fc2": np.zeros(C),
            "ln1_w": np.ones(C), "ln1_b": np.zeros(C), "ln2_w": np.ones(C), "ln2_b": np.zeros(C),
        }
    else:
        q = {
            "w_fc1": rng.normal(0.0, C ** -0.5, (hidden, C)),
            "w_fc2": rng.normal(0.0, hidden ** -0.5, (C, hidden)),
            "b_fc1": rng.normal(0.0, 0.1, hidden), "b_fc2": rng.normal(0.0, 0.1, C),
            "ln1_w": 1.0 + rng.normal(0.0, 0.1, C), "ln1_b": rng.normal(0.0, 0.1, C),
            "ln2_w": 1.0 + rng.normal(0.0, 0.1, C), "ln2_b": rng.normal(0.0, 0.1, C),
        }
    p.update({k: v.astype(np.float32) for k, v in q.items()})
    return p


def activations(B, H, W, C, seed):
    """(x, dy) ~ N(0,1), fp32, drawn in that order."""
    rng = np.random.default_rng(seed)
    x = rng.normal(0.0, 1.0, (B, H, W, C)).astype(np.float32)
    dy = rng.normal(0.0, 1.0, (B, H, W, C)).astype(np.float32)
    return x, dy


def to_bf16_bits(a):
    """Round fp32 values to bfloat16 (nearest, ties to even); returns the uint16 patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(bits):
    """Widen bfloat16 bit patterns to fp32 exactly."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(a, dtype):
    """Value the storage type ``dtype`` ('f32' or 'bf16') holds for ``a``, as fp32."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return from_bf16_bits(to_bf16_bits(a)).reshape(np.shape(a))
    raise ValueError(f"unknown dtype {dtype!r}")


# The benchmark shapes.  "layers" lists the shift of each layer of the case.
CONFIGS = {
    "c1": dict(B=1, H=16, W=16, C=60, heads=6, groups=(2,), window=8, layers=(4,), dtype="f32"),
    "c2": dict(B=32, H=64, W=64, C=60, heads=6, groups=(1, 2, 3, 6), window=8, layers=(0, 4),
               dtype="bf16"),
    "c3": dict(B=16, H=64, W=64, C=180, heads=6, groups=(1, 2, 3), window=8, layers=(0, 4),
               dtype="bf16"),
    "c4": dict(B=32, H=64, W=64, C=180, heads=6, groups=(2,), window=8,
               layers=tuple(4 * (i % 2) for i in range(36)), dtype="bf16"),
    "c5_m8": dict(B=1, H=512, W=512, C=180, heads=6, groups=(2,), window=8, layers=(4,),
                  dtype="bf16"),
    "c5_m16": dict(B=1, H=512, W=512, C=180, heads=6, groups=(2,), window=16, layers=(8,),
                   dtype="bf16"),
}
# Narrow q/k and 12x12 windows (Sec. "Parameter Allocation", Sec. "Experimental Settings"): C = 60,
# q and k of 16 resp. 32 channels in total over 4 heads (dqk = 4, 8), and 6 heads with dqk = 4,
# on 48x48 patches (the 64x64 patches of the plain cases are not a multiple of 12).
CONFIGS.update({
    "agile_h4_qk16": dict(B=32, H=48, W=48, C=60, heads=4, groups=(1, 2, 4), window=12, dqk=4,
                          layers=(0, 6), dtype="bf16"),
    "agile_h4_qk32": dict(B=32, H=48, W=48, C=60, heads=4, groups=(1, 2, 4), window=12, dqk=8,
                          layers=(0, 6), dtype="bf16"),
    "agile_h6_qk24": dict(B=32, H=48, W=48, C=60, heads=6, groups=(1, 2, 3, 6), window=12, dqk=4,
                          layers=(0, 6), dtype="bf16"),
    # forward only on a large map, as at deployment (528 = 44 windows of 12)
    "agile_infer": dict(B=1, H=528, W=528, C=60, heads=4, groups=(1, 2), window=12, dqk=4, layers=(6,),
                        dtype="bf16", forward_only=True),
})
# Whole layers (Eq. 4-5: LayerNorm, attention, MLP, skips) at the same shapes; the hidden layer of
# the MLP is twice as wide as the map, as in the lightweight Swin-family restoration networks.
CONFIGS.update({
    "astl_c2": dict(CONFIGS["c2"], block=True, hidden=120, groups=(1, 2, 3, 6)),
    "astl_agile": dict(CONFIGS["agile_h4_qk16"], block=True, hidden=120),
    "astl_c3": dict(CONFIGS["c3"], block=True, hidden=360),
    # forward only on a large map, as at deployment
    "astl_infer": dict(CONFIGS["agile_infer"], block=True, hidden=120),
    # the deep feature extractor's depth: 36 layers (6 blocks of 6), shifts 0, 4, 0, 4, ...
    "astl_stack36": dict(CONFIGS["c2"], block=True, hidden=120, stack=36, stack_shift=4, groups=(1, 2, 3, 6)),
    "astl_agile_stack36": dict(CONFIGS["agile_h4_qk16"], block=True, hidden=120, stack=36, stack_shift=6),
    # inference of one block of six whole layers on large maps (forward only)
    "astl_infer_stack6": dict(CONFIGS["c5_m8"], block=True, hidden=360, stack=6, stack_shift=4, forward_only=True),
    "astl_infer_stack6_2k": dict(CONFIGS["c5_m8"], H=2048, W=2048, block=True, hidden=360, stack=6, stack_shift=4,
                                 forward_only=True),
})
ACT_SEED = 0
LAYER_SEED0 = 100
