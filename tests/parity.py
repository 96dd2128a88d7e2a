"""Shared driver of the GPU parity tests: same seeded inputs to the HIP library and to the
CPU oracle, compared tensor by tensor.

Tolerance (stated by the benchmark definition): per output tensor
    max|gpu - oracle| / max|oracle|  <=  1e-5 for fp32,  2e-2 for bf16.
For bf16 the oracle is fed the bf16-rounded inputs, so the comparison measures the kernels'
arithmetic and the rounding of their outputs only.
"""
import numpy as np

from paper_2409_06206_amd import synth

TOL = {"f32": 1e-5, "bf16": 2e-2}
GRAD_NAMES = ("dx", "dw_qkv", "db_qkv", "dw_proj", "db_proj", "dtable")


def rel_err(got, want):
    denom = float(np.abs(want).max())
    num = float(np.abs(np.asarray(got, dtype=np.float64) - want).max())
    if denom == 0.0:
        return num
    return num / denom


def border_tokens(H, W, window, shift):
    """Boolean [H, W] map of the tokens that fall into the last window row or column of the shifted
    frame: the windows that carry the shift mask (empty when shift == 0)."""
    m = np.zeros((H, W), dtype=bool)
    if shift > 0:
        rows = (np.arange(H) - shift) % H >= H - window
        cols = (np.arange(W) - shift) % W >= W - window
        m = rows[:, None] | cols[None, :]
    return m


def border_errs(got, want, window, shift):
    """Errors of y and dx restricted to the masked windows' tokens, on those tokens' own scale: a wrong
    mask would otherwise hide under the maximum of the whole tensor."""
    out = {}
    B, H, W, C = want["y"].shape
    m = border_tokens(H, W, window, shift)
    if m.any():
        for k in ("y", "dx"):
            if k in want:
                out[k + "@masked windows"] = rel_err(np.asarray(got[k])[:, m, :], want[k][:, m, :])
    return out


def make_inputs(B, H, W, C, heads, groups, window, dtype, seed, regime, dqk=0):
    p = synth.layer_params(C, heads, groups, window, seed, regime, dqk)
    x, dy = synth.activations(B, H, W, C, synth.ACT_SEED + seed - synth.LAYER_SEED0)
    p = {k: synth.quantize(v, dtype) for k, v in p.items()}
    return synth.quantize(x, dtype), synth.quantize(dy, dtype), p


def oracle_results(oracle, x, dy, p, heads, groups, window, shift, cascade=True, backward=True, dqk=0):
    args = (p["w_qkv"], p["b_qkv"], p["w_proj"], p["b_proj"], p["table"])
    kw = dict(heads=heads, groups=groups, window=window, shift=shift, cascade=cascade, dqk=dqk)
    out = {"y": oracle.forward(x, *args, **kw)}
    if backward:
        out.update(zip(GRAD_NAMES, oracle.backward(x, dy, *args, **kw)))
    return out


# One bf16 rounding: relative error at most 2^-9.
U_BF16 = 2.0 ** -9
# bf16 rounding stages between the inputs and a gradient on the library's bf16 paths: q, k, v, the
# probabilities and the score gradient as matrix-core operands, dO, d(q|k|v), the stored result.
# Independent stages, each moving the result like one rounding of the inputs, add in quadrature.
ROUNDINGS = 8
STAGES_FACTOR = ROUNDINGS ** 0.5


def conditioning(oracle, x, dy, p, heads, groups, window, shift, cascade=True, dqk=0, probes=2):
    """How far each output of the EXACT layer moves, on the scale of its own maximum, when every
    input element is perturbed by one bf16 rounding (relative 2^-9, random signs): the tensor's
    condition number times the unit round-off, measured on the oracle alone."""
    want = oracle_results(oracle, x, dy, p, heads, groups, window, shift, cascade, True, dqk)
    worst = {k: 0.0 for k in want}
    for seed in range(probes):
        rng = np.random.default_rng(9000 + seed)
        jig = lambda a: a * (1.0 + U_BF16 * rng.choice([-1.0, 1.0], size=np.shape(a)))
        moved = oracle_results(oracle, jig(x), jig(dy), {k: jig(v) for k, v in p.items()}, heads, groups,
                               window, shift, cascade, True, dqk)
        for k in want:
            worst[k] = max(worst[k], rel_err(moved[k], want[k]))
    return worst


def gpu_results(x, dy, p, heads, groups, window, shift, dtype, cascade=True, backward=True,
                extra_flags=0, dqk=0):
    from paper_2409_06206_amd import gswa, runner
    B, H, W, C = x.shape
    flags = (0 if cascade else gswa.GSWA_NO_CASCADE) | extra_flags
    layer = runner.DeviceLayer(B, H, W, C, heads, groups, window, shift, dtype, flags, dqk=dqk)
    layer.set_params(p)
    layer.set_inputs(x, dy)
    layer.forward(keep=backward)
    if backward:
        layer.backward()
    import torch
    torch.cuda.synchronize()
    res = layer.results()
    if not backward:
        res = {"y": res["y"]}
    return res, layer


def check_case(oracle, B, H, W, C, heads, groups, window, shift, dtype, seed=synth.LAYER_SEED0,
               regime="init", cascade=True, backward=True, extra_flags=0, dqk=0, conditioned=False):
    """Every output against the oracle at the stated tolerance.  `conditioned` (bf16, tiny layers whose
    sums have too few terms for rounding noise to average out): a tensor whose exact value itself
    moves by more than TOL / sqrt(ROUNDINGS) under one bf16 rounding of every input is held to
    sqrt(ROUNDINGS) x that movement instead -- a bound computed per case and per tensor from the
    oracle alone (its condition number times the unit round-off)."""
    x, dy, p = make_inputs(B, H, W, C, heads, groups, window, dtype, seed, regime, dqk)
    want = oracle_results(oracle, x, dy, p, heads, groups, window, shift, cascade, backward, dqk)
    got, layer = gpu_results(x, dy, p, heads, groups, window, shift, dtype, cascade, backward,
                             extra_flags, dqk)
    errs = {k: rel_err(got[k], want[k]) for k in want}
    errs.update(border_errs(got, want, window, shift))
    tol = {k: TOL[dtype] for k in errs}
    if conditioned and dtype == "bf16" and backward:
        cond = conditioning(oracle, x, dy, p, heads, groups, window, shift, cascade, dqk)
        for k, c in cond.items():
            tol[k] = max(tol[k], STAGES_FACTOR * c)
    bad = {k: (e, tol[k]) for k, e in errs.items() if not e <= tol[k]}
    assert not bad, f"relative max-norm error above its bound (error, bound): {bad} (all: {errs})"
    return errs, layer


def check_block(oracle, B, H, W, C, heads, groups, window, shift, dtype, hidden, seed=synth.LAYER_SEED0,
                regime="stress", backward=True, tol_scale=1.0, extra_flags=0, dqk=0, eps=1e-5, cascade=True):
    """Whole layer (Eq. 4-5): ``oracle`` is the astl_oracle module."""
    from paper_2409_06206_amd import runner
    import torch
    p = synth.astl_params(C, heads, groups, window, hidden, seed, regime, dqk)
    x, dy = synth.activations(B, H, W, C, synth.ACT_SEED + seed - synth.LAYER_SEED0)
    p = {k: synth.quantize(v, dtype) for k, v in p.items()}
    x, dy = synth.quantize(x, dtype), synth.quantize(dy, dtype)
    kw = dict(heads=heads, groups=groups, window=window, shift=shift, eps=eps, dqk=dqk, cascade=cascade)
    if not cascade:
        from paper_2409_06206_amd import gswa
        extra_flags |= gswa.GSWA_NO_CASCADE
    want = {"y": oracle.forward(x, p, **kw)}
    if backward:
        dx, g = oracle.backward(x, dy, p, **kw)
        want["dx"] = dx
        want.update({"d" + k: v for k, v in g.items()})
    blk = runner.DeviceBlock(B, H, W, C, heads, groups, window, shift, dtype, hidden, eps, extra_flags, dqk=dqk)
    blk.set_params(p)
    blk.set_inputs(x, dy)
    blk.forward(keep=backward)
    if backward:
        blk.backward()
    torch.cuda.synchronize()
    got = blk.results()
    errs = {k: rel_err(got[k], want[k]) for k in want}
    bad = {k: e for k, e in errs.items() if not e <= TOL[dtype] * tol_scale}
    assert not bad, f"relative max-norm error above {TOL[dtype] * tol_scale}: {bad} (all: {errs})"
    return errs, blk
