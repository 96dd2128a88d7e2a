"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest

from paper_2409_06206_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


# B, H, W, C, heads, groups, window, shift, dtype, regime
SMALL = [
    (1, 16, 16, 60, 6, 2, 8, 4, "f32", "init"),      # the fp32 parity configuration
    (1, 16, 16, 60, 6, 2, 8, 4, "f32", "stress"),
    (2, 16, 24, 60, 6, 1, 8, 0, "f32", "stress"),
    (2, 24, 16, 60, 6, 3, 8, 3, "f32", "stress"),
    (1, 16, 16, 60, 6, 6, 8, 7, "f32", "stress"),
    (3, 8, 16, 12, 6, 2, 4, 1, "f32", "stress"),     # ragged: 12 channels, 16-token windows
    (1, 8, 8, 6, 3, 3, 8, 5, "f32", "stress"),       # one window per image
    (1, 7, 14, 6, 2, 1, 7, 3, "f32", "stress"),      # odd window side
    (1, 16, 16, 180, 6, 1, 8, 4, "f32", "stress"),
    (1, 16, 16, 180, 6, 3, 8, 4, "f32", "stress"),
    (1, 32, 32, 180, 6, 2, 16, 8, "f32", "stress"),  # 256-token windows
    (2, 16, 16, 60, 6, 1, 8, 0, "bf16", "init"),
    (2, 16, 16, 60, 6, 2, 8, 4, "bf16", "init"),
    (2, 16, 16, 60, 6, 2, 8, 4, "bf16", "stress"),
    (2, 24, 16, 60, 6, 3, 8, 4, "bf16", "stress"),
    (1, 16, 16, 60, 6, 6, 8, 4, "bf16", "stress"),
    (1, 16, 24, 180, 6, 1, 8, 4, "bf16", "stress"),
    (1, 16, 16, 180, 6, 2, 8, 0, "bf16", "stress"),
    (1, 16, 16, 180, 6, 3, 8, 4, "bf16", "init"),
    (1, 32, 32, 180, 6, 2, 16, 8, "bf16", "stress"),
]


@pytest.mark.parametrize("B,H,W,C,heads,groups,window,shift,dtype,regime", SMALL)
def test_small_shapes_forward_backward(oracle, B, H, W, C, heads, groups, window, shift, dtype, regime):
    _say("case", B, H, W, C, heads, groups, window, shift, dtype, regime)
    errs, _ = parity.check_case(oracle, B, H, W, C, heads, groups, window, shift, dtype,
                                seed=synth.LAYER_SEED0 + 3, regime=regime)
    _say("  errors", {k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("groups,shift", [(1, 0), (2, 4), (3, 5), (6, 4)])
def test_forced_staged_path_bf16(oracle, groups, shift):
    """The one-kernel-per-step path stays correct where a fused kernel would normally run."""
    from paper_2409_06206_amd import gswa
    parity.check_case(oracle, 2, 16, 24, 60, 6, groups, 8, shift, "bf16", regime="stress",
                      extra_flags=gswa.GSWA_FORCE_STAGED)


def test_forced_staged_path_wide_layer(oracle):
    from paper_2409_06206_amd import gswa
    parity.check_case(oracle, 1, 16, 24, 180, 6, 3, 8, 4, "bf16", regime="stress",
                      extra_flags=gswa.GSWA_FORCE_STAGED)


@pytest.mark.parametrize("C,heads", [(96, 6), (140, 5), (180, 6), (192, 6)])
def test_forced_staged_path_one_group_many_tokens(oracle, C, heads):
    """One group and at least 4096 tokens: the backward recomputes q|k|v (3C output columns: two or three column
    blocks of the kernel that streams the weights through LDS, the last one ragged or full) and, from 132 channels
    on, takes the input gradient on the same kernel."""
    from paper_2409_06206_amd import gswa
    parity.check_case(oracle, 1, 64, 72, C, heads, 1, 8, 4, "bf16", regime="stress",
                      extra_flags=gswa.GSWA_FORCE_STAGED)


@pytest.mark.parametrize("groups", [2, 3])
def test_no_cascade_flag_wide_layer(oracle, groups):
    """Wide fused path (C=180) with Eq. 8 switched off: no cascade input, no cascade gradient."""
    parity.check_case(oracle, 1, 16, 16, 180, 6, groups, 8, 4, "bf16", regime="stress", cascade=False)


@pytest.mark.parametrize("groups", [2, 3])
def test_accumulate_flag_on_wide_fused_path(oracle, groups):
    """Every partial-sum launch of the wide backward (per group, table, projection) adds into its output."""
    import torch
    from paper_2409_06206_amd import gswa, runner
    x, dy, p = parity.make_inputs(2, 16, 24, 180, 6, groups, 8, "bf16", synth.LAYER_SEED0 + 1, "stress")
    layer = runner.DeviceLayer(2, 16, 24, 180, 6, groups, 8, 4, "bf16", gswa.GSWA_ACCUM_WGRAD)
    layer.set_params(p)
    layer.set_inputs(x, dy)
    for g in layer.grads.values():
        g.fill_(0.5)
    layer.forward()
    layer.backward()
    layer.backward()
    torch.cuda.synchronize()
    got = layer.results()
    want = parity.oracle_results(oracle, x, dy, p, 6, groups, 8, 4)
    for k in parity.GRAD_NAMES[1:]:
        assert parity.rel_err(got[k] - 0.5, 2.0 * want[k]) <= parity.TOL["bf16"], k


def test_kernel_timing_aid_reports_the_launched_kernels():
    """gswa_profile_*: per-kernel HIP-event totals for one forward + backward."""
    import torch
    from paper_2409_06206_amd import gswa, runner
    x, dy, p = parity.make_inputs(2, 16, 16, 60, 6, 2, 8, "bf16", synth.LAYER_SEED0, "init")
    layer = runner.DeviceLayer(2, 16, 16, 60, 6, 2, 8, 4, "bf16")
    layer.set_params(p)
    layer.set_inputs(x, dy)
    gswa.gswa_profile_enable(True)
    try:
        gswa.gswa_profile_collect()
        layer.forward()
        layer.backward()
        res, dropped = gswa.gswa_profile_collect()
    finally:
        gswa.gswa_profile_enable(False)
    torch.cuda.synchronize()
    assert dropped == 0
    assert res["fused_fwd"][1] == 1 and res["fused_bwd"][1] == 2 and res["reduce_partials"][1] == 2  # one sum per head-group launch
    assert all(ms > 0 for ms, _ in res.values())
    layer.forward()
    assert gswa.gswa_profile_collect()[0] == {}


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_no_cascade_flag(oracle, dtype):
    parity.check_case(oracle, 1, 16, 16, 60, 6, 3, 8, 4, dtype, regime="stress", cascade=False)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_inference_mode_matches_training_forward(oracle, dtype):
    x, dy, p = parity.make_inputs(2, 16, 16, 60, 6, 2, 8, dtype, synth.LAYER_SEED0, "stress")
    a, _ = parity.gpu_results(x, dy, p, 6, 2, 8, 4, dtype, backward=True)
    b, _ = parity.gpu_results(x, dy, p, 6, 2, 8, 4, dtype, backward=False)
    assert np.array_equal(a["y"], b["y"])


def test_accumulate_flag_adds_into_parameter_gradients(oracle):
    import torch
    from paper_2409_06206_amd import gswa, runner
    x, dy, p = parity.make_inputs(1, 16, 16, 60, 6, 2, 8, "f32", synth.LAYER_SEED0, "stress")
    layer = runner.DeviceLayer(1, 16, 16, 60, 6, 2, 8, 4, "f32", gswa.GSWA_ACCUM_WGRAD)
    layer.set_params(p)
    layer.set_inputs(x, dy)
    for g in layer.grads.values():
        g.fill_(1.0)
    layer.forward()
    layer.backward()
    layer.backward()
    torch.cuda.synchronize()
    got = layer.results()
    want = parity.oracle_results(oracle, x, dy, p, 6, 2, 8, 4)
    for k in parity.GRAD_NAMES[1:]:
        assert parity.rel_err(got[k], 2.0 * want[k] + 1.0) <= 1e-5, k
    assert parity.rel_err(got["dx"], want["dx"]) <= 1e-5


def test_accumulate_flag_on_fused_path(oracle):
    import torch
    from paper_2409_06206_amd import gswa, runner
    x, dy, p = parity.make_inputs(2, 16, 16, 60, 6, 3, 8, "bf16", synth.LAYER_SEED0, "stress")
    layer = runner.DeviceLayer(2, 16, 16, 60, 6, 3, 8, 4, "bf16", gswa.GSWA_ACCUM_WGRAD)
    layer.set_params(p)
    layer.set_inputs(x, dy)
    for g in layer.grads.values():
        g.fill_(0.5)
    layer.forward()
    layer.backward()
    layer.backward()
    torch.cuda.synchronize()
    got = layer.results()
    want = parity.oracle_results(oracle, x, dy, p, 6, 3, 8, 4)
    for k in parity.GRAD_NAMES[1:]:
        assert parity.rel_err(got[k] - 0.5, 2.0 * want[k]) <= parity.TOL["bf16"], k


def test_accumulate_flag_with_narrow_query_key(oracle):
    """12 x 12 windows, narrow q/k (gradient copies summed at the end): two backward calls add twice."""
    import torch
    from paper_2409_06206_amd import gswa, runner
    shape = (2, 24, 24, 60, 4, 2, 12)
    x, dy, p = parity.make_inputs(*shape, "bf16", synth.LAYER_SEED0, "stress", dqk=4)
    layer = runner.DeviceLayer(*shape, 6, "bf16", gswa.GSWA_ACCUM_WGRAD, dqk=4)
    layer.set_params(p)
    layer.set_inputs(x, dy)
    for g in layer.grads.values():
        g.fill_(0.25)
    layer.forward()
    layer.backward()
    layer.backward()
    torch.cuda.synchronize()
    got = layer.results()
    want = parity.oracle_results(oracle, x, dy, p, 4, 2, 12, 6, dqk=4)
    for k in parity.GRAD_NAMES[1:]:
        assert parity.rel_err(got[k] - 0.25, 2.0 * want[k]) <= parity.TOL["bf16"], k
    assert parity.rel_err(got["dx"], want["dx"]) <= parity.TOL["bf16"]


def test_fused_path_gradients_are_run_to_run_identical():
    """The fused backward sums per-workgroup partials in a fixed order: no atomics on outputs."""
    import torch
    from paper_2409_06206_amd import runner
    x, dy, p = parity.make_inputs(4, 32, 32, 60, 6, 2, 8, "bf16", synth.LAYER_SEED0, "stress")
    layer = runner.DeviceLayer(4, 32, 32, 60, 6, 2, 8, 4, "bf16")
    layer.set_params(p)
    layer.set_inputs(x, dy)
    runs = []
    for _ in range(3):
        layer.forward()
        layer.backward()
        torch.cuda.synchronize()
        runs.append({k: v.copy() for k, v in layer.results().items()})
    for r in runs[1:]:
        for k in r:
            assert np.array_equal(r[k], runs[0][k]), k


def test_repeated_calls_reuse_buffers(oracle):
    """Two different inputs through the same buffers: the second result owes nothing to the first."""
    import torch
    from paper_2409_06206_amd import runner
    x1, dy1, p = parity.make_inputs(1, 16, 16, 60, 6, 2, 8, "bf16", synth.LAYER_SEED0, "stress")
    x2, dy2, _ = parity.make_inputs(1, 16, 16, 60, 6, 2, 8, "bf16", synth.LAYER_SEED0 + 9, "stress")
    layer = runner.DeviceLayer(1, 16, 16, 60, 6, 2, 8, 4, "bf16")
    layer.set_params(p)
    for x, dy in ((x1, dy1), (x2, dy2)):
        layer.set_inputs(x, dy)
        layer.forward()
        layer.backward()
        torch.cuda.synchronize()
        got = layer.results()
        want = parity.oracle_results(oracle, x, dy, p, 6, 2, 8, 4)
        for k in want:
            assert parity.rel_err(got[k], want[k]) <= parity.TOL["bf16"], k


FULL = [
    # name, groups, layer index: full benchmark shapes, every element compared
    ("c2", 1, 0), ("c2", 2, 1), ("c2", 3, 0), ("c2", 6, 1),
    ("c3", 1, 1), ("c3", 2, 0), ("c3", 3, 1),
    ("c4", 2, 1), ("c4", 3, 1),
    ("agile_h4_qk16", 2, 1), ("agile_h4_qk32", 4, 0), ("agile_h6_qk24", 2, 1), ("agile_h6_qk24", 3, 0),
]


@pytest.mark.parametrize("name,groups,layer", FULL)
def test_full_size_layers(oracle, name, groups, layer):
    cfg = synth.CONFIGS[name]
    _say("full", name, "G", groups, "layer", layer)
    errs, _ = parity.check_case(oracle, cfg["B"], cfg["H"], cfg["W"], cfg["C"], cfg["heads"], groups,
                                cfg["window"], cfg["layers"][layer], cfg["dtype"],
                                seed=synth.LAYER_SEED0 + layer, dqk=cfg.get("dqk", 0))
    _say("  errors", {k: f"{v:.2e}" for k, v in errs.items()})


# The benchmark's initialisation (weights of standard deviation 0.02) gives nearly uniform
# probabilities, which would hide a wrong mask, bias index or exponential: the wide layers are
# therefore also run at full size with scores of order 1-5 (`stress`), shifted.
FULL_STRESS = [("c2", 2, 1), ("c3", 1, 1), ("c3", 2, 1), ("c3", 3, 1), ("c4", 2, 1), ("c4", 3, 1)]


@pytest.mark.parametrize("name,groups,layer", FULL_STRESS)
def test_full_size_layers_peaky_softmax(oracle, name, groups, layer):
    cfg = synth.CONFIGS[name]
    assert cfg["layers"][layer] > 0
    _say("full, stress", name, "G", groups, "layer", layer)
    errs, _ = parity.check_case(oracle, cfg["B"], cfg["H"], cfg["W"], cfg["C"], cfg["heads"], groups,
                                cfg["window"], cfg["layers"][layer], cfg["dtype"],
                                seed=synth.LAYER_SEED0 + 40 + layer, regime="stress")
    _say("  errors", {k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("groups", [2, 3])
def test_more_windows_than_wavefronts(oracle, groups):
    """48 x (9 x 5) = 2160 windows: more than the 2048 wavefronts a forward launch has on 256
    compute units, so some waves take a second window; odd window counts per image, shifted."""
    _say("many windows", groups)
    errs, _ = parity.check_case(oracle, 48, 72, 40, 60, 6, groups, 8, 4, "bf16",
                                seed=synth.LAYER_SEED0 + 3, regime="stress")
    _say("  errors", {k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("groups", [2, 3])
def test_wide_layers_more_windows_than_wavefronts(oracle, groups):
    """27 x (9 x 5) = 1215 windows of a wide layer: more than the 1024 wavefronts of a backward launch
    on 256 compute units (a ragged second round), an odd number of windows (the kernel that takes
    them in pairs is left with one), odd window counts per image, shifted."""
    _say("many windows, wide", groups)
    errs, _ = parity.check_case(oracle, 27, 72, 40, 180, 6, groups, 8, 4, "bf16",
                                seed=synth.LAYER_SEED0 + 5, regime="stress")
    _say("  errors", {k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("shift", [2, 3, 6])
def test_wide_layers_other_shifts(oracle, shift):
    """Shifts other than half a window: even ones split the last window column's rows at a
    16-byte boundary (the streamed backward), odd ones take the per-chunk kernels."""
    parity.check_case(oracle, 1, 24, 16, 180, 6, 2, 8, shift, "bf16", regime="stress")


@pytest.mark.parametrize("regime", ["init", "stress"])
@pytest.mark.parametrize("name", ["c5_m8", "c5_m16"])
def test_large_image_inference(oracle, name, regime):
    cfg = synth.CONFIGS[name]
    _say("full", name, regime)
    errs, _ = parity.check_case(oracle, cfg["B"], cfg["H"], cfg["W"], cfg["C"], cfg["heads"],
                                cfg["groups"][0], cfg["window"], cfg["layers"][0], cfg["dtype"],
                                backward=False, regime=regime)
    _say("  errors", {k: f"{v:.2e}" for k, v in errs.items()})


def _random_shapes(n, seed):
    """Seeded random layer shapes that satisfy the divisibility rules (staged path territory)."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        M = int(rng.choice([2, 3, 4, 5, 6, 8]))
        heads = int(rng.choice([1, 2, 3, 4, 6]))
        groups = int(rng.choice([g for g in (1, 2, 3, 4, 6) if heads % g == 0]))
        d = int(rng.integers(1, 9))
        B, nh, nw = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        s = int(rng.integers(0, M))
        out.append((B, nh * M, nw * M, heads * d, heads, groups, M, s))
    return out


AGILE_SMALL = [
    # B, H, W, C, heads, groups, window, shift, dqk, dtype, regime   (Sec. "Parameter Allocation")
    (2, 24, 24, 60, 4, 2, 12, 6, 4, "f32", "stress"),
    (1, 24, 36, 60, 4, 2, 12, 0, 8, "f32", "init"),
    (2, 24, 24, 60, 6, 2, 12, 6, 4, "bf16", "stress"),
    (1, 36, 24, 60, 6, 3, 12, 5, 16, "bf16", "stress"),
    (3, 16, 24, 60, 6, 2, 8, 4, 4, "bf16", "stress"),     # narrow q/k on 8 x 8 windows
    (2, 16, 16, 60, 6, 1, 8, 4, 16, "bf16", "init"),      # q/k wider than v
    (1, 24, 24, 180, 6, 2, 12, 6, 8, "bf16", "stress"),
    (1, 16, 16, 12, 6, 6, 4, 1, 1, "f32", "stress"),
    (2, 24, 24, 60, 4, 2, 12, 6, 20, "bf16", "stress"),   # q/k of 17..32 channels: two 16-channel tiles
    (1, 24, 24, 180, 6, 3, 12, 7, 32, "bf16", "stress"),
    (2, 16, 16, 42, 6, 2, 8, 3, 5, "bf16", "stress"),     # head width 7, 21 channels per group (odd row strides)
    (1, 24, 24, 18, 6, 2, 12, 6, 3, "bf16", "stress"),    # head width 3
    (2, 24, 24, 60, 6, 1, 12, 6, 4, "bf16", "stress"),    # one group: two q/k tiles, four v tiles, two K steps
    (1, 24, 36, 60, 6, 3, 12, 5, 4, "bf16", "stress"),
    (1, 24, 24, 60, 6, 6, 12, 6, 8, "bf16", "stress"),    # one head per group
    (2, 16, 16, 60, 4, 1, 8, 4, 8, "bf16", "stress"),
    (1, 24, 24, 36, 6, 3, 12, 6, 6, "bf16", "init"),      # q/k as wide as v, spelled out
]


@pytest.mark.parametrize("B,H,W,C,heads,groups,window,shift,dqk,dtype,regime", AGILE_SMALL)
def test_narrow_query_key_and_window_12(oracle, B, H, W, C, heads, groups, window, shift, dqk, dtype, regime):
    """q and k of dqk channels per head, 12 x 12 windows: forward and every gradient."""
    parity.check_case(oracle, B, H, W, C, heads, groups, window, shift, dtype, regime=regime, dqk=dqk)
    parity.check_case(oracle, B, H, W, C, heads, groups, window, shift, dtype, regime=regime, dqk=dqk,
               cascade=False, seed=synth.LAYER_SEED0 + 3)


def test_window_forward_inference_and_staged_forward_agree(oracle):
    """12 x 12 windows, narrow q/k: the one-launch forward without a saved buffer gives the bits of the
    training forward, and the one-kernel-per-step forward the same result within the tolerance."""
    from paper_2409_06206_amd import gswa
    shape = (2, 24, 24, 60, 4, 2, 12)
    x, dy, p = parity.make_inputs(*shape, "bf16", synth.LAYER_SEED0, "stress", dqk=4)
    a, _ = parity.gpu_results(x, dy, p, 4, 2, 12, 6, "bf16", backward=True, dqk=4)
    b, _ = parity.gpu_results(x, dy, p, 4, 2, 12, 6, "bf16", backward=False, dqk=4)
    c, _ = parity.gpu_results(x, dy, p, 4, 2, 12, 6, "bf16", backward=False, dqk=4,
                              extra_flags=gswa.GSWA_FORCE_STAGED)
    assert np.array_equal(a["y"], b["y"])
    assert parity.rel_err(c["y"], a["y"].astype(np.float64)) <= parity.TOL["bf16"]


def test_spelled_out_query_key_width_takes_the_same_path(oracle):
    """dqk = C / heads is the plain layer: same kernels, same bits."""
    x, dy, p = parity.make_inputs(2, 16, 16, 60, 6, 2, 8, "bf16", synth.LAYER_SEED0, "stress")
    a, _ = parity.gpu_results(x, dy, p, 6, 2, 8, 4, "bf16")
    b, _ = parity.gpu_results(x, dy, p, 6, 2, 8, 4, "bf16", dqk=10)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


@pytest.mark.parametrize("shape", _random_shapes(16, 2024))
def test_random_shapes_fp32(oracle, shape):
    B, H, W, C, heads, groups, M, s = shape
    _say("random", shape)
    parity.check_case(oracle, B, H, W, C, heads, groups, M, s, "f32", seed=synth.LAYER_SEED0 + 7,
                      regime="stress")


@pytest.mark.parametrize("shape", _random_shapes(6, 77))
def test_random_shapes_bf16(oracle, shape):
    B, H, W, C, heads, groups, M, s = shape
    _say("random bf16", shape)
    # tiny layers (a few windows, head width down to 1): see check_case on `conditioned`
    errs, _ = parity.check_case(oracle, B, H, W, C, heads, groups, M, s, "bf16", seed=synth.LAYER_SEED0 + 8,
                                regime="stress", conditioned=True)
    _say("  errors", {k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("dtype,shape,flags", [
    ("f32", (4, 32, 32, 60, 6, 2, 8, 4), 0),                 # one-kernel-per-step path, vector ALUs
    ("f32", (2, 32, 48, 180, 6, 3, 16, 8), 0),               # 256-token windows: strips of queries
    ("bf16", (4, 32, 32, 60, 6, 2, 8, 4), "staged"),         # the same path on the matrix cores
    ("bf16", (2, 48, 48, 60, 4, 2, 12, 6), 0),               # 12 x 12 windows, narrow q/k
])
def test_reproducible_mode_gives_the_same_bits_every_run(oracle, dtype, shape, flags):
    """GSWA_DETERMINISTIC: no gradient depends on the order in which workgroups finish."""
    import torch
    from paper_2409_06206_amd import gswa, runner
    B, H, W, C, heads, groups, window, shift = shape
    dqk = 4 if window == 12 else 0
    fl = gswa.GSWA_DETERMINISTIC | (gswa.GSWA_FORCE_STAGED if flags == "staged" else 0)
    x, dy, p = parity.make_inputs(B, H, W, C, heads, groups, window, dtype, synth.LAYER_SEED0 + 5, "stress", dqk)
    layer = runner.DeviceLayer(B, H, W, C, heads, groups, window, shift, dtype, fl, dqk=dqk)
    layer.set_params(p)
    layer.set_inputs(x, dy)
    runs = []
    for _ in range(3):
        layer.ws.fill_(0x5a)          # whatever an earlier call left in the scratch must not matter
        layer.forward()
        layer.backward()
        torch.cuda.synchronize()
        runs.append({k: v.copy() for k, v in layer.results().items()})
    for r in runs[1:]:
        for k in r:
            assert np.array_equal(r[k], runs[0][k]), k
    want = parity.oracle_results(oracle, x, dy, p, heads, groups, window, shift, dqk=dqk)
    for k in want:
        assert parity.rel_err(runs[0][k], want[k]) <= parity.TOL[dtype], k


def test_training_forward_on_the_fused_path_needs_no_scratch(oracle):
    """Where gswa_query_bytes reports 0 bytes of forward scratch, ws may be NULL."""
    import torch
    from paper_2409_06206_amd import gswa, runner
    x, dy, p = parity.make_inputs(2, 16, 16, 60, 6, 2, 8, "bf16", synth.LAYER_SEED0, "stress")
    layer = runner.DeviceLayer(2, 16, 16, 60, 6, 2, 8, 4, "bf16")
    assert layer.fwd_ws_bytes == 0
    layer.set_params(p)
    layer.set_inputs(x, dy)
    layer.forward()
    torch.cuda.synchronize()
    y_ref = layer.y.clone()
    layer.y.zero_()
    q = layer.params
    gswa.gswa_forward(layer.desc, layer.x, q["w_qkv"], q["b_qkv"], q["w_proj"], q["b_proj"], q["table"],
                      layer.y, layer.saved, None)
    torch.cuda.synchronize()
    assert torch.equal(layer.y, y_ref)
    with pytest.raises(gswa.GswaError):   # inference keeps its state in the scratch: NULL is an error there
        gswa.gswa_forward(layer.desc, layer.x, q["w_qkv"], q["b_qkv"], q["w_proj"], q["b_proj"], q["table"],
                          layer.y, None, None)
