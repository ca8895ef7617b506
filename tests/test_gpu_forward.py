"""GPU parity of rocket_transform against the CPU oracle (needs an MI355X).
Every call goes through the C ABI; inputs are the seeded workloads."""
import numpy as np
import pytest

import oracle
import synth
from paper_2301_08527_amd import rocket
from kernels_of import sampled
from parity import check_forward, planes

pytestmark = pytest.mark.gpu


def _gpu(x):
    import torch
    return torch.from_numpy(x).cuda()


def _run(h, x, mask, lam=10.0, shift=-3.0):
    import torch
    out = rocket.rocket_transform(h, _gpu(x), mask, lam, shift)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _kernels(i, K=None):
    cfg = synth.CONFIGS[i]
    K = cfg["K"] if K is None else K
    # the oracle computes with kernels from its own sampler, checked equal to the library's
    return sampled(synth.seed_k(i), K, cfg["C"], cfg["L"])


def test_config0_all_masks():
    """univariate tiny, every kernel and series, every feature mask"""
    cfg = synth.CONFIGS[0]
    x = synth.make_input(0)
    h, kr = _kernels(0)
    for mask in range(1, 8):
        print("config0 mask", mask, flush=True)
        out = _run(h, x, mask)
        assert out.shape == (cfg["B"], rocket.rocket_num_features(mask) * cfg["K"])
        check_forward(x, kr, out, mask)


def test_config1_univariate_standard():
    """B=256, L=1000, K=10,000, all three features; every series and kernel"""
    cfg = synth.CONFIGS[1]
    x = synth.make_input(1)
    h, kr = _kernels(1)
    print("config1 run", flush=True)
    out = _run(h, x, cfg["features"])
    check_forward(x, kr, out, cfg["features"])


def test_config2_multivariate_full_size():
    """B=64 x 20 x 50,000, K=10,000 in the launch shape the benchmark times;
    the oracle checks every series on a dilation-stratified kernel sample."""
    cfg = synth.CONFIGS[2]
    x = synth.make_input(2)
    h, kr = _kernels(2)
    print("config2 run", flush=True)
    out = _run(h, x, cfg["features"])
    sel = synth.pick_kernels(kr, 256, seed=2)
    check_forward(x, kr, out, cfg["features"], sel=sel)
    # properties that hold for every output
    pl = planes(out.astype(np.float64), cfg["features"], cfg["K"])
    assert np.all((pl["ppv"] >= 0) & (pl["ppv"] <= 1)) and np.all(np.isfinite(pl["max"]))


def test_config4_long_series_with_spikes():
    """B=8 x 20 x 200,000, K=20,000 (dilations up to ~33,000), all features"""
    cfg = synth.CONFIGS[4]
    x = synth.make_input(4)
    h, kr = _kernels(4)
    print("config4 run", flush=True)
    out = _run(h, x, cfg["features"])
    sel = synth.pick_kernels(kr, 200, seed=4)
    check_forward(x, kr, out, cfg["features"], sel=sel)


@pytest.mark.parametrize("lam,shift", [(0.0, -3.0), (1.0, -3.0), (3.0, -3.0), (100.0, -3.0), (1e4, -3.0), (10.0, 3.0)])
def test_lambda_and_shift_sweep(lam, shift):
    rng = np.random.default_rng(21)
    B, C, L, K = 5, 7, 3001, 300
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(99, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    out = _run(h, x, 7, lam, shift)
    check_forward(x, kr, out, 7, lam=lam, shift=shift)


@pytest.mark.parametrize("B,C,L,K", [(1, 1, 11, 40), (3, 2, 12, 40), (2, 9, 64, 100), (1, 20, 257, 150),
                                     (2, 3, 1025, 120), (1, 12, 4099, 120), (2, 2, 8192, 100), (2, 2, 8193, 100),
                                     (1, 5, 12289, 160), (1, 3, 20011, 160),
                                     (8, 2, 9001, 60), (11, 3, 9000, 40), (17, 1, 16385, 30)])
def test_small_and_ragged_shapes(B, C, L, K):
    """shortest legal series, lengths that are not multiples of any tile, one series;
    lengths on both sides of the switch between the one-wavefront kernel (L <= 8192)
    and the four-wavefront kernel; batches of 8 and more series that are not multiples of
    the number of XCDs (the per-XCD series mapping leaves workgroups without a series)"""
    rng = np.random.default_rng(L)
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(7, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    out = _run(h, x, 7)
    check_forward(x, kr, out, 7)


@pytest.mark.parametrize("L", [2000, 9000])
def test_imported_extreme_kernels(L):
    """hand-built kernels: every length at d=1 and at the largest dilation,
    padded and not, single output position, nine channels; once per forward kernel"""
    rng = np.random.default_rng(5)
    C, B = 9, 3
    specs = []
    for ln in (7, 9, 11):
        dmax = (L - 1) // (ln - 1)
        for d in sorted({d for d in (1, 2, 3, 7, 8, 15, 16, 17, 63, 64, 65, 100, 255, 256, 257, dmax // 3, dmax - 1, dmax)
                         if 1 <= d <= dmax}):
            for padded in (False, True):
                nch = int(rng.integers(1, 10))
                specs.append((ln, d, padded, nch))
    length = np.array([s[0] for s in specs], np.int32)
    dil = np.array([s[1] for s in specs], np.int32)
    pad = np.array([(s[0] - 1) * s[1] // 2 if s[2] else 0 for s in specs], np.int32)
    nch = np.array([s[3] for s in specs], np.int32)
    chans = np.concatenate([rng.permutation(C)[:m] for m in nch]).astype(np.int32)
    w = rng.standard_normal(int((nch * length).sum())).astype(np.float32)
    bias = rng.uniform(-1, 1, len(specs)).astype(np.float32)
    h = rocket.rocket_kernels_import(len(specs), C, L, length, dil, pad, bias, nch, chans, w)
    kr = rocket.rocket_kernels_view_get(h)
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    out = _run(h, x, 7)
    ref = check_forward(x, kr, out, 7)
    assert ref["n_out"].min() <= 8      # some kernels have only a handful of positions


def test_constant_series_closed_form():
    """mean-centred weights: a constant series through unpadded kernels gives the bias"""
    C, L, K = 4, 900, 200
    x = np.repeat(np.array([0.5, -1.0, 2.0, 0.0], np.float32)[None, :, None], L, axis=2)
    h = rocket.rocket_make_kernels(3, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    out = planes(_run(h, x, 7).astype(np.float64), 7, K)
    un = kr["padding"] == 0
    b = kr["bias"].astype(np.float64)
    assert np.all(np.abs(out["max"][0, un] - b[un]) < 1e-5)
    clear = un & (np.abs(b) > 1e-4)
    assert np.array_equal(out["ppv"][0, clear], (b[clear] > 0).astype(np.float64))
    assert np.all(np.abs(out["softppv"][0, un] - 1 / (1 + np.exp(-(10 * b[un] - 3)))) < 1e-4)


def test_outputs_are_overwritten_and_repeatable():
    import torch
    x = synth.make_input(0)
    h, kr = _kernels(0)
    xd = _gpu(x)
    out = torch.full((16, 1000), float("nan"), device="cuda")
    ws = torch.empty(rocket.rocket_workspace_bytes(h, 16, 3), dtype=torch.uint8, device="cuda")
    ws.fill_(255)
    rocket.rocket_transform(h, xd, 3, out=out, workspace=ws)
    a = out.cpu().numpy().copy()
    rocket.rocket_transform(h, xd, 3, out=out, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(a, out.cpu().numpy()) and np.all(np.isfinite(a))
    # a side stream works as well
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        out2 = rocket.rocket_transform(h, xd, 3, workspace=ws, stream=s)
    s.synchronize()
    assert np.array_equal(a, out2.cpu().numpy())


def test_more_than_nine_channels_forward_only():
    """imported kernels may list more than nine channels: the forward pass takes them,
    the backward pass rejects them with ROCKET_ESHAPE"""
    import torch
    rng = np.random.default_rng(6)
    C, L, B, K = 14, 9001, 2, 24
    length = rng.choice([7, 9, 11], K).astype(np.int32)
    dil = rng.integers(1, 200, K).astype(np.int32)
    pad = np.where(rng.integers(0, 2, K) == 1, (length - 1) * dil // 2, 0).astype(np.int32)
    nch = rng.integers(10, C + 1, K).astype(np.int32)
    chans = np.concatenate([rng.permutation(C)[:m] for m in nch]).astype(np.int32)
    w = rng.standard_normal(int((nch * length).sum())).astype(np.float32)
    bias = rng.uniform(-1, 1, K).astype(np.float32)
    h = rocket.rocket_kernels_import(K, C, L, length, dil, pad, bias, nch, chans, w)
    kr = rocket.rocket_kernels_view_get(h)
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    check_forward(x, kr, _run(h, x, 7), 7)
    with pytest.raises(rocket.RocketError) as e:
        rocket.rocket_soft_ppv_backward(h, _gpu(x), 4, torch.zeros(B, K, device="cuda"))
    assert e.value.code == rocket.ROCKET_ESHAPE


def test_shape_mismatch_is_an_error():
    h, _ = _kernels(0)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_transform(h, _gpu(np.zeros((2, 1, 500), np.float32)), 3)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_transform(h, _gpu(np.zeros((2, 2, 512), np.float32)), 3)


def test_very_long_series_forward_and_backward():
    """one series of 3,000,000 samples: dilations up to ~375,000 (a dozen rows of that many columns),
    padding up to ~1.5 M zeros on either side, ~180 time tiles per kernel"""
    import torch
    L, C, K = 3_000_000, 2, 32
    rng = np.random.default_rng(1)
    x = rng.standard_normal((1, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(7, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    assert kr["dilation"].max() > 100_000
    print("3M-sample forward", flush=True)
    out = _run(h, x, 7)
    check_forward(x, kr, out, 7)
    from parity import check_backward
    g = rng.standard_normal((1, 3 * K)).astype(np.float32)
    print("3M-sample backward", flush=True)
    gw, gb = rocket.rocket_soft_ppv_backward(h, _gpu(x), 7, _gpu(g), 10.0, -3.0, False)
    torch.cuda.synchronize()
    check_backward(x, kr, gw.cpu().numpy(), gb.cpu().numpy(), g[:, 2 * K:], None, 10.0, -3.0)


def test_transform_can_be_captured_in_a_graph():
    """After the first call on a handle the transform only launches kernels (no allocation, no
    copy, no synchronisation), so a stream capture records it; every replay must give the
    eager result for the input that is in the captured buffer at that time."""
    import torch
    cfg = synth.CONFIGS[0]
    h, kr = _kernels(0)
    mask = 7
    xs = [synth.make_input(0), synth.make_input(0)[::-1].copy(), 0.5 * synth.make_input(0)]
    x = _gpu(xs[0])
    out = torch.empty((cfg["B"], 3 * cfg["K"]), dtype=torch.float32, device="cuda")
    ws = torch.empty(rocket.rocket_workspace_bytes(h, cfg["B"], mask), dtype=torch.uint8, device="cuda")
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        rocket.rocket_transform(h, x, mask, out=out, workspace=ws)       # first use: uploads the parameters
    s.synchronize()
    graph = torch.cuda.CUDAGraph()
    print("capturing", flush=True)
    with torch.cuda.graph(graph, stream=s):
        rocket.rocket_transform(h, x, mask, out=out, workspace=ws)
    for i, xi in enumerate(xs):
        x.copy_(_gpu(xi))
        out.fill_(-1.0)
        torch.cuda.synchronize()
        print("replay", i, flush=True)
        graph.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy().copy()
        eager = rocket.rocket_transform(h, x, mask)
        torch.cuda.synchronize()
        assert np.array_equal(got, eager.cpu().numpy())
        check_forward(xi, kr, got, mask)


def test_unit_calibration_runs_and_its_two_conv_strips_agree():
    """rocket_calibrate_units measures the units that bound the kernels; its conv strip exists in a vector form
    and a matrix (4x4x1 Toeplitz) form, and the call fails unless the two give the same outputs bit for bit"""
    u = rocket.rocket_calibrate_units()
    assert set(u) == set(rocket.CAL_NAMES)
    for name, v in u.items():
        assert np.isfinite(v) and v > 0, name
    assert 0.4 < u["mfma_valu_serial_ratio"] < 1.2
    assert u["conv_strip_valu_TFLOPs"] < 157.3 and u["conv_strip_mfma_toeplitz_TFLOPs"] < 157.3
