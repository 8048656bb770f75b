"""The entry point that allocates nothing: percentile calibration with its select state in a static device array,
against the entry point that takes a workspace, through the C ABI.  Two calls in a row on one GPU, the second on a
smaller input (the array keeps the first call's contents); results must agree to the bit, and with the oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import paper_2507_14811_amd as sq  # noqa: E402
from paper_2507_14811_amd import workloads as wl  # noqa: E402

DEV = "cuda:0"

CASES = [
    # first call: many K-segments, ragged rows; second call: fewer rows, fewer and other segments, other dtype
    (dict(M=301, K=1024, kseg=[0, 128, 384, 1024], dual=[1, 0, 1], x_dtype="bf16", p=0.999),
     dict(M=37, K=256, kseg=[0, 256], dual=[1], x_dtype="f32", p=0.99)),
    (dict(M=129, K=100, kseg=[0, 37, 100], dual=[0, 1], x_dtype="f32", p=0.9),
     dict(M=5, K=96, kseg=[0, 32, 96], dual=[1, 1], x_dtype="bf16", p=1.0)),
]


def _run(oracle, case, seed):
    M, K = case["M"], case["K"]
    w = wl.random_layer(M, K, 4, case["kseg"], [0, 4], case["dual"], seed=seed, x_dtype=case["x_dtype"], act="gelu")
    S = w.S
    if case["x_dtype"] == "bf16":
        xd = torch.from_numpy(wl.f32_to_bf16_bits(w.x).view(np.int16)).view(torch.bfloat16).to(DEV)
    else:
        xd = torch.from_numpy(w.x).to(DEV)
    layer = sq.Layer.from_workload(w)
    ws = torch.full((sq.sq_calibrate_workspace_bytes(),), 0xA5, dtype=torch.uint8, device=DEV)
    out = {}
    for name in ("workspace", "static"):
        amax = torch.full((2, S), float("nan"), dtype=torch.float32, device=DEV)
        steps = torch.full((2, S), float("nan"), dtype=torch.float32, device=DEV)
        for accumulate in (False, True):          # a fresh batch, then the same batch folded into the running maxima
            if name == "workspace":
                sq.sq_calibrate_act_percentile(layer, xd, case["p"], amax, steps, ws, accumulate=accumulate)
            else:
                sq.sq_calibrate_act_percentile_static(layer, xd, case["p"], amax, steps, accumulate=accumulate)
        torch.cuda.synchronize()
        out[name] = (amax.cpu().numpy().copy(), steps.cpu().numpy().copy())
    assert np.array_equal(out["static"][0].view(np.uint32), out["workspace"][0].view(np.uint32))
    assert np.array_equal(out["static"][1].view(np.uint32), out["workspace"][1].view(np.uint32))
    r = oracle.calibrate_act_percentile(w.x, case["kseg"], case["dual"], case["p"])
    assert np.array_equal(out["static"][1].view(np.uint32), np.stack([r[0], r[1]]).view(np.uint32))


@pytest.mark.parametrize("pair", CASES)
def test_static_scratch_percentile_two_calls_in_a_row(oracle, pair):
    sq.load_library()
    _run(oracle, pair[0], seed=101)
    _run(oracle, pair[1], seed=202)       # smaller input, right after: nothing of the first call may leak


def test_static_scratch_rejects_beyond_its_limits():
    lib = sq.load_library()
    assert lib.sq_calibrate_static_scratch_bytes() == sq.sq_calibrate_workspace_bytes() == 132608
    S = 65                                 # one K-segment more than the scratch array (and the library) holds
    layer = sq.Layer(4, S * 8, 4, [8 * i for i in range(S + 1)], [0, 4], [1] * S, [1.0] * S, [1.0] * S)
    x = torch.zeros((4, S * 8), dtype=torch.float32, device=DEV)
    a = torch.zeros((2, S), dtype=torch.float32, device=DEV)
    with pytest.raises(sq.SqError) as e:
        sq.sq_calibrate_act_percentile_static(layer, x, 0.5, a, a.clone())
    assert e.value.status == 2             # SQ_ERR_UNSUPPORTED, nothing launched
