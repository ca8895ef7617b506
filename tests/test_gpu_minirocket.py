"""GPU parity of the MINIROCKET-style variant (paper section 2) against the CPU oracle: the predetermined
kernel set bit for bit, the biases fitted to data within the feature tolerance, and the PPV features.
Needs an MI355X.  (Parity with the original MINIROCKET model is not claimed: see oracle/minirocket.py.)"""
import numpy as np
import pytest

import oracle
import synth
from kernels_of import INT_FIELDS
from paper_2301_08527_amd import rocket
from parity import ATOL, RTOL, check_forward

pytestmark = pytest.mark.gpu


def _gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _same_set(h, kr):
    v = rocket.rocket_kernels_view_get(h)
    for name in INT_FIELDS:
        assert np.array_equal(v[name], kr[name]), name
    assert np.array_equal(v["weights"], kr["weights"])
    return v


@pytest.mark.parametrize("seed,groups,C,L", [(1, 3, 1, 9), (2, 5, 4, 700), (3, 40, 20, 50000), (2**64 - 2, 2, 12, 8193)])
def test_kernel_set_is_the_oracles(seed, groups, C, L):
    h = rocket.rocket_minirocket_kernels(seed, groups, C, L)
    v = _same_set(h, oracle.minirocket_kernels(seed, groups, C, L))
    assert np.all(v["bias"] == 0) and len(v["length"]) == 84 * groups


def _fit_and_check(seed, groups, x):
    import torch
    B, C, L = x.shape
    h = rocket.rocket_minirocket_kernels(seed, groups, C, L)
    kr0 = oracle.minirocket_kernels(seed, groups, C, L)
    print("minirocket fit", x.shape, groups, flush=True)
    rocket.rocket_minirocket_fit_bias(h, _gpu(x), seed + 100)
    torch.cuda.synchronize()
    got = rocket.rocket_kernels_view_get(h)["bias"].astype(np.float64)
    kr, ex, rank = oracle.minirocket_fit_bias(x, kr0, seed + 100)
    ref = kr["bias"].astype(np.float64)
    err = np.abs(got - ref)
    assert np.all(err <= RTOL * np.abs(ref) + ATOL), (int(np.argmax(err)), float(err.max()))
    return h, kr


def test_bias_fit_and_features_small():
    rng = np.random.default_rng(71)
    x = rng.standard_normal((5, 3, 1200)).astype(np.float32)
    h, kr = _fit_and_check(5, 4, x)
    import torch
    xt = rng.standard_normal((7, 3, 1200)).astype(np.float32)
    out = rocket.rocket_transform(h, _gpu(xt), 2)
    torch.cuda.synchronize()
    # the library's biases differ from the oracle's by rounding: compare the features through the oracle's kernels
    # with the library's biases, so that both sides pool the same thing
    kr_lib = dict(kr)
    kr_lib["bias"] = rocket.rocket_kernels_view_get(h)["bias"]
    check_forward(xt, kr_lib, out.cpu().numpy(), 2)
    # and on the training batch every kernel's PPV on its own example is what the rank says (up to near-ties)
    out_train = rocket.rocket_transform(h, _gpu(x), 2).cpu().numpy().astype(np.float64)
    ref = oracle.minirocket_transform(x, kr_lib)
    assert np.all(np.abs(np.rint(out_train * ref["n_out"][None, :]) - ref["count"]) <= ref["ambiguous"])


def test_bias_fit_with_ties_and_one_series():
    """8-bit-like samples (many equal outputs: the selected order statistic is still an element of the row) and a
    training batch of one series, shortest legal length included"""
    rng = np.random.default_rng(72)
    x = rng.integers(0, 4, size=(1, 2, 333)).astype(np.float32)
    _fit_and_check(6, 2, x)
    _fit_and_check(7, 1, rng.standard_normal((2, 1, 9)).astype(np.float32))
    _fit_and_check(8, 2, rng.standard_normal((3, 5, 64)).astype(np.float32))


def test_paper_shape_sample():
    """20 channels x 50,000 samples, 119 groups (9,996 kernels): fit on 4 series, features of 3 others, a
    stratified sample of kernels checked by the oracle"""
    import torch
    x = synth.make_input(2, B=7)
    groups = 119
    h = rocket.rocket_minirocket_kernels(31, groups, 20, 50000)
    kr0 = oracle.minirocket_kernels(31, groups, 20, 50000)
    _same_set(h, kr0)
    print("minirocket paper shape: fit", flush=True)
    rocket.rocket_minirocket_fit_bias(h, _gpu(x[:4]), 77)
    torch.cuda.synchronize()
    bias = rocket.rocket_kernels_view_get(h)["bias"]
    sel = synth.pick_kernels(kr0, 96, seed=5)
    ex, q = oracle.minirocket.bias_draws(77, kr0["K"], 4)
    for k in sel:
        y = oracle.conv_output(x[ex[k]], kr0, int(k))
        r = int(np.floor(q[k] * (len(y) - 1)))
        ref = -np.partition(y, r)[r]
        assert abs(float(bias[k]) - ref) <= RTOL * abs(ref) + ATOL, int(k)
    print("minirocket paper shape: transform", flush=True)
    out = rocket.rocket_transform(h, _gpu(x[4:]), 2)
    torch.cuda.synchronize()
    kr_lib = dict(kr0)
    kr_lib["bias"] = bias
    check_forward(x[4:], kr_lib, out.cpu().numpy(), 2, sel=sel)
    print("minirocket paper shape: group kernel", flush=True)
    fast = rocket.rocket_minirocket_transform(h, _gpu(x[4:]))
    torch.cuda.synchronize()
    check_forward(x[4:], kr_lib, fast.cpu().numpy(), 2, sel=sel)
    # a batch of eight, as the benchmark launches it (one series per XCD); its first three rows are those above
    x8 = np.concatenate([x[4:], synth.make_input(2, B=12)[7:]])
    fast8 = rocket.rocket_minirocket_transform(h, _gpu(x8))
    torch.cuda.synchronize()
    assert torch.equal(fast8[:3], fast)
    check_forward(x8, kr_lib, fast8.cpu().numpy(), 2, sel=sel[::4], rows=np.arange(3, 8))


# ---------------------------------------------------------------- the group kernel (rocket_minirocket_transform)

def _group_transform_case(seed, groups, B, C, L, fitted):
    """features of rocket_minirocket_transform against the oracle (integer counts, the usual PPV rule) and
    against rocket_transform's PPV plane on the same handle (different rounding order: same rule)"""
    import torch
    print("minirocket group kernel", seed, groups, B, C, L, fitted, flush=True)
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    if L >= 64:
        x += np.sin(np.arange(L, dtype=np.float32) * (6.28318 / 37.0))[None, None, :]     # correlated neighbours, as in real series
    h = rocket.rocket_minirocket_kernels(seed, groups, C, L)
    kr = oracle.minirocket_kernels(seed, groups, C, L)
    if fitted:
        rocket.rocket_minirocket_fit_bias(h, _gpu(x[: max(1, B // 2)]), seed + 9)
        torch.cuda.synchronize()
    else:
        rocket.rocket_kernels_set_params(h, None, rng.uniform(-2.0, 2.0, kr["K"]).astype(np.float32))
    out = rocket.rocket_minirocket_transform(h, _gpu(x))
    plain = rocket.rocket_transform(h, _gpu(x), 2)
    torch.cuda.synchronize()
    kr = dict(kr)
    kr["bias"] = rocket.rocket_kernels_view_get(h)["bias"]
    assert out.shape == (B, kr["K"])
    ref = check_forward(x, kr, out.cpu().numpy(), 2)
    n = ref["n_out"][None, :].astype(np.float64)
    diff = np.abs(np.rint(out.cpu().numpy().astype(np.float64) * n) - np.rint(plain.cpu().numpy().astype(np.float64) * n))
    assert np.all(diff <= 2 * ref["ambiguous"])
    return h, x, out


@pytest.mark.parametrize("seed,groups,B,C,L,fitted", [
    (11, 1, 1, 1, 9, False),          # one output position (or nine with padding)
    (12, 3, 2, 2, 10, False),
    (13, 6, 3, 3, 73, True),
    (14, 12, 8, 4, 1000, True),       # eight series: the per-XCD series mapping
    (15, 10, 5, 20, 4105, False),     # dilations on either side of 256: tiles of consecutive positions and tiles of rows x columns
    (16, 30, 3, 6, 9000, True),       # many groups of either kind, ragged last row
    (17, 24, 8, 9, 20011, False),
    (18, 8, 1, 2, 200001, True),      # long series: dilations up to 25,000, a hundred column blocks to a row
])
def test_group_kernel_matches_oracle(seed, groups, B, C, L, fitted):
    _group_transform_case(seed, groups, B, C, L, fitted)


def test_group_kernel_covers_both_tile_kinds():
    """the sizes above do reach both kinds of work item (checked on the kernels, not assumed)"""
    for seed, groups, C, L in [(16, 30, 6, 9000), (17, 24, 9, 20011)]:
        d = oracle.minirocket_kernels(seed, groups, C, L)["dilation"][::84]
        assert (d <= 256).any() and (d > 256).any() and (d > 1024).any() == (L > 10000)


def test_group_kernel_is_deterministic_and_reusable():
    import torch
    h, x, out = _group_transform_case(21, 8, 8, 5, 3000, True)
    ws = torch.empty(rocket.rocket_minirocket_workspace_bytes(h, 8), dtype=torch.uint8, device="cuda")
    ws.fill_(0xAB)                      # the call may not rely on what the workspace held
    again = rocket.rocket_minirocket_transform(h, _gpu(x), workspace=ws)
    small = rocket.rocket_minirocket_transform(h, _gpu(x[:3]), workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out, again) and torch.equal(out[:3], small)


def test_group_kernel_argument_errors():
    import torch
    x = torch.zeros(2, 3, 100, device="cuda")
    plain = rocket.rocket_make_kernels(1, 84, 3, 100)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_minirocket_transform(plain, x)
    h = rocket.rocket_minirocket_kernels(1, 2, 3, 100)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_minirocket_transform(h, x, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    rocket.rocket_minirocket_transform(h, x)
    w = rocket.rocket_kernels_view_get(h)["weights"].copy()
    rocket.rocket_kernels_set_params(h, w, None)          # weights touched: no longer known to be the predetermined set
    assert rocket.rocket_minirocket_workspace_bytes(h, 2) == 0
    with pytest.raises(rocket.RocketError):
        rocket.rocket_minirocket_transform(h, x)
    rocket.rocket_transform(h, x, 2)                      # the general path still serves it
    torch.cuda.synchronize()


def test_group_kernel_can_be_captured_in_a_graph():
    """after its first call on a handle the group transform only launches kernels (the counters are cleared by
    a kernel, not a memset), so a stream capture records it; every replay must give the eager result for the
    input that is in the captured buffer at that time"""
    import torch
    rng = np.random.default_rng(33)
    B, C, L, groups = 8, 3, 2500, 6
    h = rocket.rocket_minirocket_kernels(33, groups, C, L)
    rocket.rocket_kernels_set_params(h, None, rng.uniform(-1.0, 1.0, 84 * groups).astype(np.float32))
    xs = [rng.standard_normal((B, C, L)).astype(np.float32) for _ in range(3)]
    x = _gpu(xs[0])
    out = torch.empty((B, 84 * groups), dtype=torch.float32, device="cuda")
    ws = torch.empty(rocket.rocket_minirocket_workspace_bytes(h, B), dtype=torch.uint8, device="cuda")
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        rocket.rocket_minirocket_transform(h, x, out=out, workspace=ws)   # first use: uploads parameters and work items
    s.synchronize()
    graph = torch.cuda.CUDAGraph()
    print("capturing", flush=True)
    with torch.cuda.graph(graph, stream=s):
        rocket.rocket_minirocket_transform(h, x, out=out, workspace=ws)
    for i, xi in enumerate(xs):
        x.copy_(_gpu(xi))
        out.fill_(-1.0)
        torch.cuda.synchronize()
        print("replay", i, flush=True)
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        eager = rocket.rocket_minirocket_transform(h, x)
        torch.cuda.synchronize()
        assert torch.equal(got, eager)


def test_group_kernel_from_bytes():
    """rocket_minirocket_transform_u8: raw 8-bit samples, z-normalised inside the call, against the oracle's
    z-scores through the oracle's transform; a constant row and a saturated row included"""
    import torch
    rng = np.random.default_rng(44)
    B, C, L, groups = 4, 5, 3001, 10
    raw = rng.integers(60, 200, size=(B, C, L)).astype(np.uint8)
    raw[1, 2, :] = 77                      # zero variance: becomes zeros
    raw[2, 0, :] = np.where(rng.random(L) < 0.5, 0, 255).astype(np.uint8)
    h = rocket.rocket_minirocket_kernels(44, groups, C, L)
    kr = oracle.minirocket_kernels(44, groups, C, L)
    rocket.rocket_kernels_set_params(h, None, rng.uniform(-1.5, 1.5, kr["K"]).astype(np.float32))
    out = rocket.rocket_minirocket_transform_u8(h, _gpu(raw))
    torch.cuda.synchronize()
    kr = dict(kr)
    kr["bias"] = rocket.rocket_kernels_view_get(h)["bias"]
    check_forward(oracle.znormalize_u8(raw), kr, out.cpu().numpy(), 2)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_minirocket_transform_u8(h, _gpu(raw.astype(np.float32)))
