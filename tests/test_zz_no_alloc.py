"""gswa_backward_static (the backward for callers that cannot allocate or pass a workspace)
against gswa_backward, through the C ABI: two calls in a row, the second on a smaller layer,
each compared with the ordinary entry point on the same inputs and with the CPU oracle."""
import numpy as np
import pytest

from paper_2409_06206_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu


def _static_backward(layer):
    from paper_2409_06206_amd import gswa
    p, g = layer.params, layer.grads
    gswa.gswa_backward_static(layer.desc, layer.x, layer.dy, p["w_qkv"], p["b_qkv"], p["w_proj"],
                              p["b_proj"], p["table"], layer.saved, layer.dx, g["w_qkv"], g["b_qkv"],
                              g["w_proj"], g["b_proj"], g["table"])


def _run_pair(oracle, shape, dtype, exact):
    """Ordinary backward, then the static one on the same layer object (outputs cleared in between)."""
    import torch
    from paper_2409_06206_amd import runner
    B, H, W, C, heads, groups, window, shift = shape
    x, dy, p = parity.make_inputs(B, H, W, C, heads, groups, window, dtype, synth.LAYER_SEED0 + 7, "stress")
    want = parity.oracle_results(oracle, x, dy, p, heads, groups, window, shift)
    layer = runner.DeviceLayer(B, H, W, C, heads, groups, window, shift, dtype)
    layer.set_params(p)
    layer.set_inputs(x, dy)
    layer.forward()
    layer.backward()
    torch.cuda.synchronize()
    ref = layer.results()
    layer.dx.zero_()
    for t in layer.grads.values():
        t.fill_(float("nan"))
    _static_backward(layer)
    torch.cuda.synchronize()
    got = layer.results()
    for k in parity.GRAD_NAMES:
        assert np.isfinite(got[k]).all(), k
        if exact:   # the fused path sums in a fixed order: same bits from both entry points
            assert np.array_equal(got[k], ref[k]), k
        else:       # fp32 atomics: the order of the additions differs from run to run
            assert parity.rel_err(got[k], ref[k].astype(np.float64)) <= parity.TOL[dtype], k
        assert parity.rel_err(got[k], want[k]) <= parity.TOL[dtype], k


@pytest.mark.parametrize("dtype,first,second,exact", [
    # fused path (per-workgroup partial sums in the scratch): larger, then smaller
    ("bf16", (4, 32, 32, 60, 6, 2, 8, 4), (1, 16, 16, 60, 6, 2, 8, 4), True),
    # staged path (q|k|v, its gradient and the gradient copies in the scratch)
    ("f32", (2, 16, 24, 60, 6, 2, 8, 4), (1, 16, 16, 60, 6, 2, 8, 4), False),
])
def test_two_calls_in_a_row_second_smaller(oracle, dtype, first, second, exact):
    print("static backward", dtype, first, "then", second, flush=True)
    _run_pair(oracle, first, dtype, exact)
    _run_pair(oracle, second, dtype, exact)


def test_rejects_layers_beyond_the_built_in_scratch():
    from paper_2409_06206_amd import gswa, runner
    import torch
    # staged fp32 layer whose scratch (two q|k|v buffers of T x 3C floats) exceeds the limit
    desc = gswa.make_desc(64, 64, 64, 60, 6, 1, 8, 0, "f32")
    _, _, bwd = gswa.gswa_query_bytes(desc)
    assert bwd > gswa.GSWA_STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    with pytest.raises(gswa.GswaError) as e:
        gswa.gswa_backward_static(desc, *([dummy] * 14))
    assert e.value.status == gswa.GSWA_ETOOBIG
