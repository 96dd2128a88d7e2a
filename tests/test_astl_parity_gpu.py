"""GPU parity of the whole layer (Eq. 4-5: LayerNorm, attention, MLP, skips) through the C ABI
against the fp64 oracle, element by element on the same seeded inputs.  Tolerance as for the
attention layer: max-norm relative error per tensor, 1e-5 in fp32 and 2e-2 in bf16."""
import numpy as np
import pytest

from oracle import astl_oracle
from paper_2409_06206_amd import gswa, synth
from tests import parity

pytestmark = pytest.mark.gpu

SMALL = [
    # fp32: vector and scalar channel layouts of the per-token kernels, several row passes
    dict(B=1, H=16, W=16, C=60, heads=6, groups=2, window=8, shift=4, dtype="f32", hidden=120),
    dict(B=2, H=8, W=8, C=12, heads=2, groups=1, window=4, shift=0, dtype="f32", hidden=20),
    dict(B=1, H=8, W=12, C=6, heads=2, groups=2, window=4, shift=1, dtype="f32", hidden=9),
    dict(B=1, H=8, W=8, C=68, heads=4, groups=2, window=4, shift=2, dtype="f32", hidden=100),
    dict(B=1, H=8, W=8, C=200, heads=4, groups=1, window=4, shift=2, dtype="f32", hidden=64),
    dict(B=1, H=8, W=8, C=66, heads=6, groups=3, window=4, shift=0, dtype="f32", hidden=40),
    # bf16: the benchmark's channel counts, every group setting, both window sizes
    dict(B=2, H=16, W=16, C=60, heads=6, groups=1, window=8, shift=0, dtype="bf16", hidden=120),
    dict(B=2, H=16, W=16, C=60, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=120),
    dict(B=3, H=16, W=24, C=60, heads=6, groups=3, window=8, shift=4, dtype="bf16", hidden=120),
    dict(B=1, H=16, W=16, C=60, heads=6, groups=6, window=8, shift=0, dtype="bf16", hidden=120),
    dict(B=1, H=24, W=24, C=60, heads=4, groups=2, window=12, shift=6, dtype="bf16", hidden=120, dqk=4),
    dict(B=1, H=16, W=16, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360),
    dict(B=1, H=8, W=8, C=30, heads=3, groups=1, window=4, shift=2, dtype="bf16", hidden=50),
    dict(B=1, H=16, W=16, C=60, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=60),
    dict(B=5, H=8, W=8, C=60, heads=6, groups=2, window=8, shift=0, dtype="bf16", hidden=128),
]


def _id(c):
    return "-".join(f"{k}{v}" for k, v in c.items())


@pytest.mark.parametrize("case", SMALL, ids=_id)
def test_layer_matches_oracle(case):
    print("case", case, flush=True)
    parity.check_block(astl_oracle, **case)


@pytest.mark.parametrize("case", [SMALL[0], SMALL[7], SMALL[10]], ids=_id)
def test_init_regime(case):
    """Identity LayerNorms, small weights: the skip path dominates y, the gradients still have to match."""
    print("case", case, flush=True)
    parity.check_block(astl_oracle, regime="init", **case)


@pytest.mark.parametrize("case", [SMALL[7], SMALL[10]], ids=_id)
def test_every_path_of_the_attention_layer(case):
    print("case", case, flush=True)
    parity.check_block(astl_oracle, extra_flags=gswa.GSWA_FORCE_STAGED, **case)


@pytest.mark.parametrize("case", [SMALL[0], SMALL[7], SMALL[11]], ids=_id)
def test_inference_call_gives_the_training_output(case):
    print("case", case, flush=True)
    import torch
    _, blk = parity.check_block(astl_oracle, backward=False, **case)
    y_inf = blk.y.clone()
    blk.forward(keep=True)
    torch.cuda.synchronize()
    assert torch.equal(y_inf, blk.y)


@pytest.mark.parametrize("case", [
    SMALL[0], SMALL[7],
    # a wide layer with enough tokens for the streaming weight-gradient kernel, whose sum then writes or adds
    # straight into the gradients of the two MLP maps
    dict(B=4, H=64, W=64, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360),
], ids=_id)
def test_accumulate_flag_adds_into_every_parameter_gradient(case):
    print("case", case, flush=True)
    import torch
    _, blk = parity.check_block(astl_oracle, **case)
    first = {k: v.clone() for k, v in blk.grads.items()}
    from paper_2409_06206_amd import astl
    c = dict(case)
    blk.desc = astl.make_desc(c["B"], c["H"], c["W"], c["C"], c["heads"], c["groups"], c["window"], c["shift"],
                              c["dtype"], c["hidden"], flags=gswa.GSWA_ACCUM_WGRAD, dqk=c.get("dqk", 0))
    blk.backward()
    torch.cuda.synchronize()
    for k, v in blk.grads.items():
        want = 2.0 * first[k]
        err = float((v - want).abs().max()) / max(float(want.abs().max()), 1e-30)
        assert err <= 1e-3, (k, err)


@pytest.mark.parametrize("name", ["astl_c2", "astl_agile", "astl_c3"])
def test_benchmark_shape_pair_against_the_oracle(name):
    """The two layers of a whole-layer workload at its full size, every output element."""
    cfg = synth.CONFIGS[name]
    for li, shift in enumerate(cfg["layers"]):
        case = dict(B=cfg["B"], H=cfg["H"], W=cfg["W"], C=cfg["C"], heads=cfg["heads"], groups=2,
                    window=cfg["window"], shift=shift, dtype=cfg["dtype"], hidden=cfg["hidden"],
                    dqk=cfg.get("dqk", 0))
        print("case", case, flush=True)
        parity.check_block(astl_oracle, seed=synth.LAYER_SEED0 + li, **case)


@pytest.mark.parametrize("case", [
    dict(B=2, H=64, W=32, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360),
    # 4800 tokens: 37 passes of 128 and a ragged one
    dict(B=3, H=40, W=40, C=180, heads=6, groups=3, window=8, shift=0, dtype="bf16", hidden=360),
    dict(B=4, H=64, W=64, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360),
], ids=_id)
def test_wide_layer_with_enough_tokens_for_the_streaming_weight_gradients(case):
    """C = 180, hidden 360 from 4096 tokens on (the scratch is everything behind h | dpre in the workspace):
    the MLP's four weight gradients come from ONE launch of the kernel that streams the rows once and sums
    per-workgroup partial arrays in a fixed order, straight into the gradients."""
    import torch
    print("case", case, flush=True)
    gswa.gswa_profile_enable(True)
    gswa.gswa_profile_collect()
    parity.check_block(astl_oracle, **case)
    torch.cuda.synchronize()
    names, dropped = gswa.gswa_profile_collect()
    gswa.gswa_profile_enable(False)
    assert dropped == 0
    assert names["fc_wgrad"][1] == 1 and "fill_zero" not in names, names


def test_wide_layer_with_few_tokens_keeps_the_gradient_copies():
    """2048 tokens: too few rows for the streaming weight-gradient kernel (it takes 4096 and more); the layer
    takes the kernels that add into 16 gradient copies (and still the streaming MLP kernels)."""
    import torch
    case = dict(B=1, H=64, W=32, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360)
    print("case", case, flush=True)
    gswa.gswa_profile_enable(True)
    gswa.gswa_profile_collect()
    parity.check_block(astl_oracle, **case)
    torch.cuda.synchronize()
    names, dropped = gswa.gswa_profile_collect()
    gswa.gswa_profile_enable(False)
    assert dropped == 0
    assert names["fc_wgrad"][1] == 2 and "fill_zero" in names and "mlp_bwd" in names, names


@pytest.mark.parametrize("case,kernels", [
    # hidden 400 > 384: the first map (180 -> 400) keeps its whole weight matrix in LDS and takes Eq. 4's skip and
    # LN_2 in its operand read and the GELU in its stores; the second (K = 400) runs on the chunked kernel
    (dict(B=1, H=64, W=64, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=400), ("fc1_linear", "fc2_linear")),
    # 256 channels > 192: both maps on the whole-matrix kernel with 512 threads (K = 256 and 288: more than six
    # steps of 32), LN_2 in the operand read of the first; ragged last 16-row tile (4160 tokens)
    (dict(B=1, H=80, W=52, C=256, heads=4, groups=2, window=4, shift=2, dtype="bf16", hidden=288), ("fc1_linear", "fc2_linear")),
], ids=lambda v: _id(v) if isinstance(v, dict) else "")
def test_wide_layers_beyond_the_streaming_mlp_kernels(case, kernels):
    """Wide bf16 layers that the streaming MLP kernels do not take (hidden > 384 or C > 192), with enough
    tokens (>= 4096) for the linear-map kernel that holds a whole weight matrix in LDS."""
    import torch
    print("case", case, flush=True)
    gswa.gswa_profile_enable(True)
    gswa.gswa_profile_collect()
    parity.check_block(astl_oracle, **case)
    torch.cuda.synchronize()
    names, dropped = gswa.gswa_profile_collect()
    gswa.gswa_profile_enable(False)
    assert dropped == 0
    assert all(k in names for k in kernels) and "mlp_fwd" not in names, names
    # LN_2 of the forward and of the backward's recomputation ride in the first map: only LN_1 is launched (twice)
    assert names["ln_fwd"][1] == 2, names


def test_wide_layer_backward_is_run_to_run_identical():
    """A wide bf16 layer with enough tokens for the streaming weight-gradient kernel sums every parameter
    gradient in a fixed order (partial vectors per workgroup, no atomics, no flag needed): two backward passes
    give the same bits."""
    import torch
    case = dict(B=4, H=64, W=64, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360)
    print("case", case, flush=True)
    _, blk = parity.check_block(astl_oracle, **case)
    first = {k: v.clone() for k, v in blk.grads.items()}
    dx = blk.dx.clone()
    for _ in range(2):
        blk.backward()
        torch.cuda.synchronize()
        assert torch.equal(blk.dx, dx)
        for k, v in blk.grads.items():
            assert torch.equal(v, first[k]), k


@pytest.mark.parametrize("case", [SMALL[0], SMALL[8]], ids=_id)
def test_groups_without_the_cascade(case):
    print("case", case, flush=True)
    parity.check_block(astl_oracle, cascade=False, **case)


@pytest.mark.parametrize("eps", [1e-6, 1e-2, 0.5])
def test_eps_enters_both_layer_norms(eps):
    """A large eps changes the result visibly; both sides must take it from the descriptor."""
    case = dict(SMALL[7])
    print("case", case, "eps", eps, flush=True)
    parity.check_block(astl_oracle, eps=eps, **case)


def test_narrow_bf16_layers_take_the_fused_mlp_kernels():
    """The kernel timing aid names what ran: one fused launch per pass for the MLP half of a narrow
    bf16 layer, the per-step kernels otherwise (fp32, wide layers, forced)."""
    import torch
    case = dict(SMALL[7])
    print("case", case, flush=True)
    for flags, fused in ((0, True), (gswa.GSWA_FORCE_STAGED, False)):
        gswa.gswa_profile_enable(True)
        gswa.gswa_profile_collect()
        parity.check_block(astl_oracle, extra_flags=flags, **case)
        torch.cuda.synchronize()
        names, dropped = gswa.gswa_profile_collect()
        gswa.gswa_profile_enable(False)
        assert dropped == 0
        assert ("mlp_fwd" in names and "mlp_bwd" in names and "ln_fwd+mlp_reduce" in names) == fused, names
        assert ("fc1_linear" in names and "gelu_fwd" in names and "fc_wgrad" in names) == (not fused), names
        assert names["ln_fwd"][1] == (1 if fused else 4) and names["ln_bwd"][1] == (1 if fused else 2), names


@pytest.mark.parametrize("C,hidden", [(64, 120), (60, 128), (32, 64), (28, 60), (16, 24)])
def test_padding_edges_of_the_fused_mlp_tiles(C, hidden):
    """Channel and hidden widths at and next to the tile sizes of the fused MLP kernels."""
    heads = 4 if C % 4 == 0 else 2
    case = dict(B=2, H=8, W=8, C=C, heads=heads, groups=2, window=4, shift=2, dtype="bf16", hidden=hidden)
    print("case", case, flush=True)
    parity.check_block(astl_oracle, **case)


@pytest.mark.parametrize("case", [
    dict(B=1, H=4, W=4, C=256, heads=4, groups=2, window=4, shift=1, dtype="f32", hidden=16),
    dict(B=1, H=4, W=8, C=256, heads=8, groups=1, window=4, shift=0, dtype="bf16", hidden=24),
    dict(B=2, H=4, W=4, C=4, heads=2, groups=2, window=2, shift=1, dtype="bf16", hidden=4),
    dict(B=2, H=4, W=4, C=8, heads=2, groups=1, window=4, shift=2, dtype="f32", hidden=7),
    dict(B=1, H=8, W=8, C=20, heads=2, groups=2, window=4, shift=0, dtype="bf16", hidden=36),
], ids=_id)
def test_extreme_widths(case):
    """The widest supported map (256 channels), the narrowest fused one, an odd hidden width."""
    print("case", case, flush=True)
    parity.check_block(astl_oracle, **case)


@pytest.mark.parametrize("C,hidden,tokens", [
    (180, 360, (1, 8, 12)),    # the benchmark's widths, 96 tokens: fewer tiles than waves of a workgroup
    (192, 384, (1, 8, 8)),     # every tile of both instantiation's largest shape full
    (132, 100, (2, 8, 12)),    # narrowest of the six-step kernel: two ragged channel steps; hidden not a multiple of 32
    (128, 256, (1, 12, 8)),    # widest of the four-step kernel, whole steps only
    (68, 32, (3, 4, 4)),       # narrowest wide layer, one stream unit, one of its three hidden steps in use
    (100, 196, (1, 20, 4)),    # the row's last four channels alone in a piece (C % 8 == 4), ragged hidden step
    (96, 384, (5, 4, 4)),
])
def test_shape_edges_of_the_streaming_mlp_forward_of_wide_layers(C, hidden, tokens):
    """Layers wider than 64 channels (up to 192, hidden up to 384) take the forward kernel that streams the
    MLP's weights through LDS: channel counts around its 32-channel steps, hidden widths around its 32-feature
    steps and 96-feature units, token counts that are not a multiple of the 16-token tiles."""
    import torch
    B, H, W = tokens
    case = dict(B=B, H=H, W=W, C=C, heads=4, groups=2, window=4, shift=1, dtype="bf16", hidden=hidden)
    print("case", case, flush=True)
    gswa.gswa_profile_enable(True)
    gswa.gswa_profile_collect()
    parity.check_block(astl_oracle, **case)
    torch.cuda.synchronize()
    names, dropped = gswa.gswa_profile_collect()
    gswa.gswa_profile_enable(False)
    assert dropped == 0
    assert "mlp_fwd" in names and "fc2_linear" not in names, names


def test_many_rounds_of_the_streaming_mlp_forward():
    """More 16-token tiles than the launch has waves (several rounds per wave, a ragged last round)."""
    case = dict(B=9, H=64, W=64, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360)
    print("case", case, flush=True)
    parity.check_block(astl_oracle, backward=False, **case)


def test_ragged_token_count_in_the_fused_mlp_kernels():
    """Token counts that are not a multiple of the 16-token tiles or of the 128-token rounds."""
    for B, H, W in ((1, 4, 12), (3, 4, 4), (7, 8, 4)):
        case = dict(B=B, H=H, W=W, C=60, heads=6, groups=2, window=4, shift=1, dtype="bf16", hidden=120)
        print("case", case, flush=True)
        parity.check_block(astl_oracle, **case)


def test_graph_replays_of_a_layer_pair_match_the_eager_result():
    """A step of two chained whole layers captured into a HIP graph: every replay, with eager work
    and synchronisation in between, gives the eager outputs (the attention layer's fused path sums
    in a fixed order; the LayerNorm gradients go through atomics, hence a tolerance there)."""
    import torch
    from paper_2409_06206_amd import runner
    cfg = dict(B=2, H=16, W=16, C=60, heads=6, groups=2, window=8, dtype="bf16", hidden=120)
    x, dy = synth.activations(cfg["B"], cfg["H"], cfg["W"], cfg["C"], 1)
    blocks = []
    for li, shift in enumerate((0, 4)):
        blk = runner.DeviceBlock(cfg["B"], cfg["H"], cfg["W"], cfg["C"], cfg["heads"], cfg["groups"], cfg["window"],
                                 shift, cfg["dtype"], cfg["hidden"])
        blk.set_params(synth.astl_params(cfg["C"], cfg["heads"], cfg["groups"], cfg["window"], cfg["hidden"],
                                         200 + li, "stress"))
        blocks.append(blk)
    blocks[0].set_inputs(x)
    blocks[1].dy = runner.to_device(dy, cfg["dtype"])
    blocks[1].x, blocks[0].dy = blocks[0].y, blocks[1].dx

    def step():
        for b in blocks:
            b.forward()
        for b in reversed(blocks):
            b.backward()

    def snapshot():
        torch.cuda.synchronize()
        out = {}
        for i, b in enumerate(blocks):
            out.update({f"{i}.{k}": v.copy() for k, v in b.results().items()})
        return out

    print("eager step", flush=True)
    step()
    want = snapshot()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    print("capture", flush=True)
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(4):
        # eager work of the program's own between the replays: the outputs are overwritten
        for b in blocks:
            b.y.zero_()
            b.dx.zero_()
            for g in b.grads.values():
                g.fill_(7.0)
        torch.cuda.synchronize()
        print("replay", rep, flush=True)
        graph.replay()
        got = snapshot()
        for k, w in want.items():
            exact = k.endswith(".y") or k.endswith(".dx")
            if exact:
                assert np.array_equal(got[k], w), (rep, k)
            else:
                assert parity.rel_err(got[k], w) <= 1e-4, (rep, k, parity.rel_err(got[k], w))


STACKS = [
    dict(B=1, H=16, W=16, C=60, heads=6, groups=2, window=8, shift=4, dtype="f32", hidden=120, n_layers=3),
    dict(B=2, H=16, W=16, C=60, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=120, n_layers=5),
    dict(B=1, H=24, W=24, C=60, heads=4, groups=2, window=12, shift=6, dtype="bf16", hidden=120, n_layers=4, dqk=4),
    # wide layers: the streaming MLP kernels (the forward one hands LN_1 to the next layer), 4096 tokens
    dict(B=1, H=64, W=64, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360, n_layers=3),
]


@pytest.mark.parametrize("every", [0, 1, 2, 3, 9])
@pytest.mark.parametrize("case", STACKS, ids=_id)
def test_stack_matches_oracle_with_and_without_checkpointing(case, every):
    """A sequence of layers with alternating shift; recomputed blocks give the same gradients."""
    import torch
    from paper_2409_06206_amd import runner
    c = dict(case)
    print("case", c, "checkpoint_every", every, flush=True)
    dtype, L, dqk = c["dtype"], c["n_layers"], c.get("dqk", 0)
    ps = [synth.astl_params(c["C"], c["heads"], c["groups"], c["window"], c["hidden"], 300 + l, "stress", dqk)
          for l in range(L)]
    ps = [{k: synth.quantize(v, dtype) for k, v in p.items()} for p in ps]
    x, dy = (synth.quantize(a, dtype) for a in synth.activations(c["B"], c["H"], c["W"], c["C"], 2))
    # a tensor handed from one layer to the next is a tensor of the layer's element type on both sides
    # ("bf16 activations with fp32 accumulation"); inside a layer the oracle stays in fp64
    kw = dict(heads=c["heads"], groups=c["groups"], window=c["window"], shift=c["shift"], dqk=dqk,
              store=None if dtype == "f32" else (lambda a: synth.quantize(a, dtype)))
    want = {"y": astl_oracle.stack_forward(x, ps, **kw)}
    dx, grads = astl_oracle.stack_backward(x, dy, ps, **kw)
    want["dx"] = dx
    for l, g in enumerate(grads):
        want.update({f"{l}.d{k}": v for k, v in g.items()})
    st = runner.DeviceStack(c["B"], c["H"], c["W"], c["C"], c["heads"], c["groups"], c["window"], c["shift"], dtype,
                            c["hidden"], L, every, dqk=dqk)
    st.set_params(ps)
    st.set_inputs(x, dy)
    st.forward()
    st.backward()
    torch.cuda.synchronize()
    got = st.results()
    tol = parity.TOL[dtype]
    errs = {k: parity.rel_err(got[k], w) for k, w in want.items()}
    bad = {k: e for k, e in errs.items() if not e <= tol}
    assert not bad, (bad, max(errs.values()))
    # inference call: same output, nothing saved
    y_train = st.y.clone()
    st.y.zero_()
    st.forward(keep=False)
    torch.cuda.synchronize()
    assert torch.equal(st.y, y_train)


TILED = [
    # (case, band sizes in window rows): bands that divide the map and bands that do not, one band per
    # image, one window row per band; shift 0 in every layer; odd shift; three images
    (dict(B=1, H=48, W=16, C=60, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=120, n_layers=4),
     (1, 2, 4, 5, 6, 9)),
    (dict(B=3, H=32, W=24, C=60, heads=6, groups=3, window=8, shift=3, dtype="bf16", hidden=120, n_layers=3),
     (1, 3)),
    (dict(B=2, H=40, W=16, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360, n_layers=3),
     (2, 3)),
    (dict(B=1, H=24, W=8, C=60, heads=6, groups=2, window=8, shift=0, dtype="bf16", hidden=120, n_layers=2),
     (1, 2)),
    (dict(B=2, H=20, W=12, C=12, heads=2, groups=1, window=4, shift=1, dtype="f32", hidden=20, n_layers=3),
     (1, 2, 4)),
    (dict(B=1, H=48, W=24, C=60, heads=4, groups=2, window=12, shift=6, dtype="bf16", hidden=120, n_layers=2,
          dqk=4), (1, 3)),
]


@pytest.mark.parametrize("case,bands", TILED, ids=lambda v: _id(v) if isinstance(v, dict) else str(v))
def test_band_by_band_inference_is_the_whole_map_inference(case, bands):
    """Bands of window rows through every layer: the oracle's output within tolerance, and the very bits of
    the call that takes each image as one band (a window's arithmetic does not depend on the band it is in)."""
    import torch
    from paper_2409_06206_amd import runner
    c = dict(case)
    print("case", c, flush=True)
    dtype, L, dqk = c["dtype"], c["n_layers"], c.get("dqk", 0)
    ps = [synth.astl_params(c["C"], c["heads"], c["groups"], c["window"], c["hidden"], 500 + l, "stress", dqk)
          for l in range(L)]
    ps = [{k: synth.quantize(v, dtype) for k, v in p.items()} for p in ps]
    x = synth.quantize(synth.activations(c["B"], c["H"], c["W"], c["C"], 1)[0], dtype)
    kw = dict(heads=c["heads"], groups=c["groups"], window=c["window"], shift=c["shift"], dqk=dqk,
              store=None if dtype == "f32" else (lambda a: synth.quantize(a, dtype)))
    want = astl_oracle.stack_forward(x, ps, **kw)
    st = runner.DeviceStack(c["B"], c["H"], c["W"], c["C"], c["heads"], c["groups"], c["window"], c["shift"], dtype,
                            c["hidden"], L, 0, dqk=dqk)
    st.set_params(ps)
    st.set_inputs(x)
    x_before = st.x.clone()
    # one band per image: every layer is one plain call of the whole-layer forward per image
    st.forward_tiled(c["H"])
    torch.cuda.synchronize()
    whole = st.y.clone()
    assert parity.rel_err(runner.to_host(whole), want) <= parity.TOL[dtype]
    for nb in bands:
        print("band_windows", nb, flush=True)
        st.y.fill_(float("nan"))
        st.forward_tiled(nb)
        torch.cuda.synchronize()
        assert torch.equal(st.y, whole), nb
        assert torch.equal(st.x, x_before)
    # the whole-map call hands LayerNorm_1 from layer to layer inside its MLP kernel where it can, which
    # sums a row in another order: equal up to the rounding of the stored activations
    st.forward(keep=False)
    torch.cuda.synchronize()
    assert parity.rel_err(runner.to_host(st.y), runner.to_host(whole)) <= (1e-6 if dtype == "f32" else 2e-2)


def test_inference_sequence_at_the_benchmark_size():
    """astl_infer_stack6 as bench.py runs it (six whole layers, one 512x512 map, C = 180, hidden 360, in one
    call): every output element against the oracle's loop over the layers, and the band-by-band form on the
    same map against both."""
    import torch
    from paper_2409_06206_amd import runner
    cfg = synth.CONFIGS["astl_infer_stack6"]
    L, groups, dtype = cfg["stack"], cfg["groups"][0], cfg["dtype"]
    print("case", cfg, flush=True)
    ps = [synth.astl_params(cfg["C"], cfg["heads"], groups, cfg["window"], cfg["hidden"], 700 + l, "stress")
          for l in range(L)]
    ps = [{k: synth.quantize(v, dtype) for k, v in p.items()} for p in ps]
    x, _ = synth.activations(cfg["B"], cfg["H"], cfg["W"], cfg["C"], synth.ACT_SEED + 9)
    x = synth.quantize(x, dtype)
    want = astl_oracle.stack_forward(x, ps, heads=cfg["heads"], groups=groups, window=cfg["window"],
                                     shift=cfg["stack_shift"], store=lambda a: synth.quantize(a, dtype))
    st = runner.DeviceStack(cfg["B"], cfg["H"], cfg["W"], cfg["C"], cfg["heads"], groups, cfg["window"],
                            cfg["stack_shift"], dtype, cfg["hidden"], L, 0, inference_only=True)
    st.set_params(ps)
    st.set_inputs(x)
    st.forward(keep=False)
    torch.cuda.synchronize()
    whole = runner.to_host(st.y)
    assert parity.rel_err(whole, want) <= parity.TOL[dtype]
    st.y.fill_(float("nan"))
    st.forward_tiled(16)
    torch.cuda.synchronize()
    banded = runner.to_host(st.y)
    assert parity.rel_err(banded, want) <= parity.TOL[dtype]
    assert parity.rel_err(banded, whole) <= parity.TOL[dtype]


def _random_layers(n, seed):
    """Seeded random whole-layer shapes that satisfy the divisibility rules: any window, head count,
    head width, hidden width, narrow or plain queries and keys."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        M = int(rng.choice([2, 3, 4, 5, 6, 8]))
        heads = int(rng.choice([1, 2, 3, 4, 6]))
        groups = int(rng.choice([g for g in (1, 2, 3, 4, 6) if heads % g == 0]))
        d = int(rng.integers(1, 11))
        if heads * d > 256:
            continue
        B, nh, nw = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        case = dict(B=B, H=nh * M, W=nw * M, C=heads * d, heads=heads, groups=groups, window=M,
                    shift=int(rng.integers(0, M)), hidden=int(rng.integers(1, 140)),
                    dqk=int(rng.choice([0, 0, 1, 3, 4])))
        # A LayerNorm over very few channels is ill-conditioned with a tiny eps: 1/sqrt(var + eps)
        # reaches eps^-1/2 = 316 when a token's channels nearly coincide, and every rounding of the
        # normalised value is amplified by that factor in both arithmetics.  Such layers get an eps
        # that conditions them (eps is a parameter of the layer): 1/sqrt(var + eps) <= 10.
        if heads * d < 6:
            case["eps"] = 1e-2
        out.append(case)
    return out


@pytest.mark.parametrize("case", _random_layers(14, 31), ids=_id)
def test_random_layers_fp32(case):
    print("case", case, flush=True)
    parity.check_block(astl_oracle, dtype="f32", **case)


@pytest.mark.parametrize("case", _random_layers(10, 32), ids=_id)
def test_random_layers_bf16(case):
    print("case", case, flush=True)
    parity.check_block(astl_oracle, dtype="bf16", **case)
