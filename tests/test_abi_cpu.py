"""Host-side checks of the C ABI that need no GPU: the library loads, exports what the header
declares, validates arguments before touching the device, and reports buffer sizes."""
import os
import re

import pytest

from paper_2409_06206_amd import gswa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="gswa.h", prefix="gswa"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(%s_[a-z_]+)\s*\(" % prefix, text)))


def test_library_exports_every_declared_symbol():
    L = gswa.lib()
    names = declared_functions()
    assert set(names) == set(gswa.EXPORTS)
    for n in names:
        assert hasattr(L, n), n
    assert gswa.gswa_version() >= 100


def test_strerror_texts():
    assert gswa.gswa_strerror(0) == "ok"
    for code in (-1, -2, -3, -99):
        assert gswa.gswa_strerror(code)


GOOD = dict(B=2, H=16, W=16, C=60, heads=6, groups=2, window=8, shift=4, dtype="bf16")


@pytest.mark.parametrize("change", [
    dict(B=0), dict(H=12), dict(W=20), dict(C=62), dict(heads=4, groups=3), dict(groups=4),
    dict(shift=8), dict(shift=-1), dict(window=0), dict(dtype=7), dict(flags=64), dict(dqk=-1),
])
def test_invalid_descriptors_are_rejected(change):
    desc = gswa.make_desc(**{**GOOD, **change})
    with pytest.raises(gswa.GswaError) as ei:
        gswa.gswa_query_bytes(desc)
    assert ei.value.status == gswa.GSWA_EINVAL


def test_null_pointers_are_rejected_before_any_launch():
    desc = gswa.make_desc(**GOOD)
    fake = 0x1000  # never dereferenced: validation fails first
    with pytest.raises(gswa.GswaError) as ei:
        gswa.gswa_forward(desc, fake, fake, fake, fake, fake, fake, None, None, fake, stream=0)
    assert ei.value.status == gswa.GSWA_EINVAL
    with pytest.raises(gswa.GswaError) as ei:
        gswa.gswa_forward(desc, fake, fake, fake, fake, fake, fake, fake, None, fake + 8, stream=0)
    assert ei.value.status == gswa.GSWA_EINVAL  # misaligned workspace
    with pytest.raises(gswa.GswaError) as ei:
        gswa.gswa_backward(desc, fake, fake, fake, fake, fake, fake, fake, None, fake, fake, fake,
                           fake, fake, fake, fake, stream=0)
    assert ei.value.status == gswa.GSWA_EINVAL
    with pytest.raises(gswa.GswaError) as ei:  # x not 16-byte aligned
        gswa.gswa_forward(desc, fake + 2, fake, fake, fake, fake, fake, 2 * fake, None, fake, stream=0)
    assert ei.value.status == gswa.GSWA_EINVAL


@pytest.mark.parametrize("dtype,e", [("f32", 4), ("bf16", 2)])
def test_saved_state_is_one_activation_and_scratch_shrinks_with_groups(dtype, e):
    """Staged path: the head-group loop bounds the scratch: one group's q|k|v (and its gradient)."""
    T, C = 2 * 16 * 16, 60
    prev = None
    for G in (1, 2, 3, 6):
        desc = gswa.make_desc(**{**GOOD, "groups": G, "dtype": dtype, "flags": gswa.GSWA_FORCE_STAGED})
        saved, fwd, bwd = gswa.gswa_query_bytes(desc)
        assert saved == T * C * e
        params = 3 * C * C // G + 3 * C + C * C + C + 15 * 15 * 6
        copies = (16 * params * 4 + 255) // 256 * 256     # parameter-gradient copies, see gswa.h
        per_window = (T // 64 * 15 * 15 * 6 * 4 + 255) // 256 * 256 if dtype == "bf16" else 0   # see gswa.h
        assert fwd == 3 * T * (C // G) * e and bwd == 2 * fwd + copies + per_window
        assert all(v % 256 == 0 for v in (saved, fwd, bwd))
        if prev is not None:
            assert saved + bwd < prev
        prev = saved + bwd


def test_narrow_query_key_sizes_the_group_scratch():
    """Sec. "Parameter Allocation": a group's q|k|v row has 2*hg*dqk + Cg features; 12 x 12 windows."""
    T, C, heads = 2 * 24 * 24, 60, 6
    for G, dqk in ((1, 4), (2, 4), (3, 8), (2, 16)):
        desc = gswa.make_desc(B=2, H=24, W=24, C=C, heads=heads, groups=G, window=12, shift=6,
                              dtype="bf16", dqk=dqk)
        saved, fwd, bwd = gswa.gswa_query_bytes(desc)
        row = 2 * (heads // G) * dqk + C // G
        assert saved == T * C * 2
        assert fwd == T * row * 2 and bwd >= 2 * fwd
    same = [gswa.gswa_query_bytes(gswa.make_desc(**{**GOOD, "dqk": q})) for q in (0, 10)]
    assert same[0][0] >= same[1][0]  # dqk = C/heads spelled out is the plain layer


def test_fused_path_sizes():
    """Fused bf16 path: the saved state is one [T, C] activation plus the packed parameters
    (independent of the batch); forward scratch is only needed for inference."""
    T, C = 2 * 16 * 16, 60
    for G in (1, 2, 3, 6):
        saved, fwd, bwd = gswa.gswa_query_bytes(gswa.make_desc(**{**GOOD, "groups": G}))
        assert T * C * 2 < saved <= T * C * 2 + 256 * 1024
        big = gswa.gswa_query_bytes(gswa.make_desc(**{**GOOD, "groups": G, "B": 8}))[0]
        assert big - 4 * T * C * 2 == saved - T * C * 2
        assert fwd == 0
        assert bwd > 0 and bwd % 256 == 0


def test_query_path_names_the_organisation_that_serves_a_layer():
    """gswa_query_path: the benchmark shapes take the fused kernels, fp32 and forced layers the per-step
    path, narrow q/k and 12 x 12 windows the one-launch forward with a per-step backward."""
    F, S, WF = gswa.GSWA_PATH_FUSED, gswa.GSWA_PATH_STAGED, gswa.GSWA_PATH_WINDOW_FWD
    assert gswa.gswa_query_path(gswa.make_desc(**GOOD)) == (F, F)
    assert gswa.gswa_query_path(gswa.make_desc(**{**GOOD, "C": 180})) == (F, F)
    assert gswa.gswa_query_path(gswa.make_desc(**{**GOOD, "dtype": "f32"})) == (S, S)
    assert gswa.gswa_query_path(gswa.make_desc(**{**GOOD, "flags": gswa.GSWA_FORCE_STAGED})) == (S, S)
    assert gswa.gswa_query_path(gswa.make_desc(**{**GOOD, "C": 180, "H": 32, "W": 32, "window": 16, "shift": 8})) == (F, S)
    assert gswa.gswa_query_path(gswa.make_desc(**{**GOOD, "dqk": 4})) == (WF, S)
    assert gswa.gswa_query_path(gswa.make_desc(B=1, H=24, W=24, C=60, heads=6, groups=2, window=12, shift=6,
                                               dtype="bf16")) == (WF, S)
    with pytest.raises(gswa.GswaError):
        gswa.gswa_query_path(gswa.make_desc(**{**GOOD, "groups": 4}))


def test_whole_layer_entry_points_are_exported():
    from paper_2409_06206_amd import astl
    names = declared_functions("astl.h", "astl")
    assert set(names) == set(astl.EXPORTS)
    L = astl.lib()
    for n in names:
        assert hasattr(L, n), n


@pytest.mark.parametrize("change", [dict(hidden=0), dict(hidden=-4), dict(eps=-1.0), dict(eps=float("nan")),
                                    dict(H=12), dict(dtype=5)])
def test_invalid_whole_layer_descriptors_are_rejected(change):
    from paper_2409_06206_amd import astl
    desc = astl.make_desc(**{**GOOD, "hidden": 120, **change})
    with pytest.raises(gswa.GswaError) as ei:
        astl.astl_query_bytes(desc)
    assert ei.value.status == gswa.GSWA_EINVAL


def test_whole_layer_rejects_wide_channels_and_null_pointers():
    from paper_2409_06206_amd import astl
    desc = astl.make_desc(**{**GOOD, "C": 264, "heads": 6, "hidden": 120})
    with pytest.raises(gswa.GswaError) as ei:
        astl.astl_query_bytes(desc)
    assert ei.value.status == gswa.GSWA_EUNSUPPORTED
    desc = astl.make_desc(**{**GOOD, "hidden": 120})
    fake = 0x1000  # never dereferenced: validation fails first
    full = {n: fake for n in astl.PARAM_FIELDS}
    with pytest.raises(gswa.GswaError) as ei:
        astl.astl_forward(desc, fake, {**full, "w_fc1": None}, fake + 0x1000, None, fake, stream=0)
    assert ei.value.status == gswa.GSWA_EINVAL
    with pytest.raises(gswa.GswaError) as ei:
        astl.astl_forward(desc, fake, full, fake + 0x1000, None, fake + 8, stream=0)
    assert ei.value.status == gswa.GSWA_EINVAL
    with pytest.raises(gswa.GswaError) as ei:
        astl.astl_backward(desc, fake, fake, full, fake, fake + 0x2000, {**full, "ln2_b": None}, fake, stream=0)
    assert ei.value.status == gswa.GSWA_EINVAL


def test_whole_layer_sizes_hold_the_attention_layers_state_and_one_activation():
    from paper_2409_06206_amd import astl
    desc = astl.make_desc(**{**GOOD, "hidden": 120})
    saved, fwd, bwd = astl.astl_query_bytes(desc)
    a_saved, a_fwd, a_bwd = gswa.gswa_query_bytes(desc.attn)
    act = 2 * 16 * 16 * 60 * 2
    assert a_saved + act <= saved <= a_saved + act + 68 * 1024  # (+ the MLP's repacked weights)
    assert fwd >= 2 * act + a_fwd and bwd >= 3 * act + a_bwd
    assert saved % 256 == 0 and fwd % 256 == 0 and bwd % 256 == 0


def test_stack_descriptor_validation_and_sizes():
    from paper_2409_06206_amd import astl
    base = dict(B=2, H=16, W=16, C=60, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=120, n_layers=12)
    for change in (dict(n_layers=0), dict(shift=8), dict(shift=-1), dict(checkpoint_every=-1), dict(hidden=0)):
        with pytest.raises(gswa.GswaError) as ei:
            astl.astl_stack_query_bytes(astl.make_stack_desc(**{**base, **change}))
        assert ei.value.status == gswa.GSWA_EINVAL, change
    layer = astl.astl_query_bytes(astl.make_desc(**{k: v for k, v in base.items() if k != "n_layers"}))
    act = 2 * 16 * 16 * 60 * 2
    keep_all = astl.astl_stack_query_bytes(astl.make_stack_desc(**base))
    assert keep_all[0] == 12 * (layer[0] + act)          # every layer's state and output
    blocks = astl.astl_stack_query_bytes(astl.make_stack_desc(**base, checkpoint_every=4))
    assert blocks[0] == 2 * act                          # the inputs of layers 4 and 8
    assert blocks[2] >= 4 * (layer[0] + act)             # one block is rebuilt in the scratch
    # at the benchmark's size recomputed blocks need far less than keeping all 36 layers
    big = dict(base, B=32, H=64, W=64, n_layers=36)
    all36 = astl.astl_stack_query_bytes(astl.make_stack_desc(**big))
    six = astl.astl_stack_query_bytes(astl.make_stack_desc(**big, checkpoint_every=6))
    assert six[0] + six[2] < 0.3 * (all36[0] + all36[2])
    # one block that spans the whole stack keeps (next to) nothing
    whole = astl.astl_stack_query_bytes(astl.make_stack_desc(**base, checkpoint_every=50))
    assert whole[0] == act
    fake = 0x1000
    full = {n: fake for n in astl.PARAM_FIELDS}
    with pytest.raises(gswa.GswaError) as ei:   # a null parameter in the last layer, found before any launch
        astl.astl_stack_forward(astl.make_stack_desc(**base), fake, [full] * 11 + [{**full, "ln1_w": None}],
                                fake + 0x1000, None, fake, stream=0)
    assert ei.value.status == gswa.GSWA_EINVAL


def test_tiled_inference_scratch_follows_the_band_not_the_map():
    """Scratch of the band-by-band inference call: set by the band, the same for any map height."""
    from paper_2409_06206_amd import astl
    base = dict(B=1, H=512, W=512, C=180, heads=6, groups=2, window=8, shift=4, dtype="bf16", hidden=360,
                n_layers=36)
    sd = astl.make_stack_desc(**base)
    for bad in (0, -3):
        with pytest.raises(gswa.GswaError) as ei:
            astl.astl_stack_tiled_query_bytes(sd, bad)
        assert ei.value.status == gswa.GSWA_EINVAL
    whole = astl.astl_stack_query_bytes(sd)[1]
    b8 = astl.astl_stack_tiled_query_bytes(sd, 8)
    b16 = astl.astl_stack_tiled_query_bytes(sd, 16)
    assert b8 % 256 == 0 and b8 < b16 < whole
    band_act = 17 * 8 * 512 * 180 * 2                     # 16 window rows and the one that is dropped
    assert 4 * band_act <= b16 <= 12 * band_act
    tall = astl.make_stack_desc(**dict(base, H=4096))
    assert astl.astl_stack_tiled_query_bytes(tall, 16) == b16
    assert astl.astl_stack_query_bytes(tall)[1] > 7 * whole
    # one band per image: as much as the whole map of one image needs, whatever the batch
    one = astl.astl_stack_tiled_query_bytes(sd, 1000)
    assert one == astl.astl_stack_tiled_query_bytes(astl.make_stack_desc(**dict(base, B=4)), 64)
    fake = 0x1000
    full = {n: fake for n in astl.PARAM_FIELDS}
    with pytest.raises(gswa.GswaError) as ei:   # x and y must differ; found before any launch
        astl.astl_stack_forward_tiled(sd, fake, [full] * 36, fake, 8, fake, stream=0)
    assert ei.value.status == gswa.GSWA_EINVAL


def _spread(n, step=1 << 28):
    """n fake device addresses far apart (never dereferenced: the calls below fail validation)."""
    return [(i + 1) * step for i in range(n)]


def test_partially_overlapping_buffers_are_rejected():
    """Outputs and scratch are checked against every other buffer as byte ranges, not as pointers."""
    desc = gswa.make_desc(**{**GOOD, "flags": gswa.GSWA_FORCE_STAGED})
    act = 2 * 16 * 16 * 60 * 2
    saved_b, fwd_b, bwd_b = gswa.gswa_query_bytes(desc)
    x, wq, bq, wp, bp, tb, y, saved, ws = _spread(9)

    def fwd(**kw):
        a = dict(x=x, w_qkv=wq, b_qkv=bq, w_proj=wp, b_proj=bp, bias_table=tb, y=y, saved=saved, ws=ws)
        a.update(kw)
        with pytest.raises(gswa.GswaError) as ei:
            gswa.gswa_forward(desc, a["x"], a["w_qkv"], a["b_qkv"], a["w_proj"], a["b_proj"], a["bias_table"],
                              a["y"], a["saved"], a["ws"], stream=0)
        assert ei.value.status == gswa.GSWA_EINVAL

    fwd(y=x + 64)                       # y starts inside x
    fwd(y=x - act + 256)                # y ends inside x
    fwd(saved=ws + fwd_b - 256)         # saved starts inside the scratch
    fwd(y=wp + 16)                      # y inside a weight
    fwd(ws=x + act - 256)               # scratch starts inside x
    fwd(ws=None)                        # this path needs scratch

    dy, dx, gwq, gbq, gwp, gbp, gtb = [a + (1 << 27) for a in _spread(7)]

    def bwd(**kw):
        a = dict(x=x, dy=dy, saved=saved, dx=dx, dw_qkv=gwq, db_qkv=gbq, dw_proj=gwp, db_proj=gbp,
                 dbias_table=gtb, ws=ws)
        a.update(kw)
        with pytest.raises(gswa.GswaError) as ei:
            gswa.gswa_backward(desc, a["x"], a["dy"], wq, bq, wp, bp, tb, a["saved"], a["dx"], a["dw_qkv"],
                               a["db_qkv"], a["dw_proj"], a["db_proj"], a["dbias_table"], a["ws"], stream=0)
        assert ei.value.status == gswa.GSWA_EINVAL

    bwd(dx=dy + 128)                    # dx starts inside dy
    bwd(dx=saved + saved_b - 16)        # dx starts in the last bytes of saved
    bwd(dw_qkv=ws + 1024)               # a gradient inside the scratch
    bwd(db_proj=gwp + 60 * 60 * 4 - 16)  # two gradients share bytes
    bwd(ws=x + 256)
    bwd(ws=None)


def test_reproducible_mode_is_a_valid_flag_and_sizes_its_scratch():
    base = gswa.gswa_query_bytes(gswa.make_desc(**{**GOOD, "dtype": "f32"}))
    det = gswa.gswa_query_bytes(gswa.make_desc(**{**GOOD, "dtype": "f32", "flags": gswa.GSWA_DETERMINISTIC}))
    assert det[0] == base[0] and det[1] == base[1]
    params = 3 * 60 * 60 // 2 + 3 * 60 + 60 * 60 + 60 + 15 * 15 * 6
    per_window = 2 * 16 * 16 // 64 * 15 * 15 * 6 * 4
    up = lambda b: (b + 255) // 256 * 256
    assert det[2] - base[2] == up(64 * params * 4) - up(16 * params * 4) + up(per_window)
    # the fused path sums in a fixed order anyway: the flag changes nothing there
    assert gswa.gswa_query_bytes(gswa.make_desc(**{**GOOD, "flags": gswa.GSWA_DETERMINISTIC})) == \
        gswa.gswa_query_bytes(gswa.make_desc(**GOOD))


def test_fused_path_memory_does_not_grow_with_the_group_count():
    """Default (fused) path at the benchmark's narrow and wide shapes: saved state plus scratch is
    non-increasing in the group count -- the scratch holds the partial parameter gradients of one
    head-group launch at a time, which shrink with the group."""
    for shape, groups in (((32, 64, 64, 60), (1, 2, 3, 6)), ((16, 64, 64, 180), (2, 3))):
        B, H, W, C = shape
        prev = None
        for G in groups:
            saved, fwd, bwd = gswa.gswa_query_bytes(gswa.make_desc(B, H, W, C, 6, G, 8, 4, "bf16"))
            assert fwd == 0 and saved >= B * H * W * C * 2
            total = saved + bwd
            if prev is not None:
                assert total <= prev, (C, G, total, prev)
            prev = total
    # narrow layers: strictly falling from one group to two and to three
    t = [sum(gswa.gswa_query_bytes(gswa.make_desc(32, 64, 64, 60, 6, G, 8, 4, "bf16"))[::2]) for G in (1, 2, 3)]
    assert t[0] > t[1] > t[2]
