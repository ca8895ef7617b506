"""GPU parity of rocket_soft_ppv_backward against the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest

import oracle
import synth
from paper_2301_08527_amd import rocket
from kernels_of import sampled
from parity import check_backward

pytestmark = pytest.mark.gpu


def _gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _backward(h, x, mask, grad_out, lam, shift, include_max):
    import torch
    gw, gb = rocket.rocket_soft_ppv_backward(h, _gpu(x), mask, _gpu(grad_out), lam, shift, include_max)
    torch.cuda.synchronize()
    return gw.cpu().numpy(), gb.cpu().numpy()


def _split(grad_out, mask, K):
    """(g_soft, g_max) planes of an upstream gradient laid out like the forward output."""
    F = rocket.rocket_num_features(mask)
    g_soft = grad_out[:, (F - 1) * K:F * K]
    g_max = grad_out[:, :K] if mask & 1 else None
    return g_soft, g_max


def _stable_argmax(x, kr, sel=None):
    """kernels whose maximum is separated from the runner-up, so fp32 and fp64 agree on where it is"""
    o = oracle.transform(x, kr, sel=sel)
    return o["gap"].min(axis=0) > 1e-3


@pytest.mark.parametrize("mask,include_max", [(4, False), (5, False), (5, True), (7, True), (6, False)])
def test_small_all_kernels(mask, include_max):
    rng = np.random.default_rng(31)
    B, C, L, K = 4, 6, 1500, 160
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(41, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    F = rocket.rocket_num_features(mask)
    grad_out = rng.standard_normal((B, F * K)).astype(np.float32)
    lam, shift = 4.0, -3.0
    print("backward small", mask, include_max, flush=True)
    gw, gb = _backward(h, x, mask, grad_out, lam, shift, include_max)
    g_soft, g_max = _split(grad_out, mask, K)
    sel = None
    if include_max:
        sel = np.nonzero(_stable_argmax(x, kr))[0].astype(np.int32)
        assert len(sel) > K // 2
    rep = {}
    check_backward(x, kr, gw, gb, g_soft, g_max if include_max else None, lam, shift, sel=sel, report=rep)
    print("worst error / bound:", rep["worst_ratio"], flush=True)


@pytest.mark.parametrize("lam,shift", [(0.0, -3.0), (1.0, -3.0), (10.0, -3.0), (100.0, -3.0), (10.0, 3.0)])
def test_lambda_sweep(lam, shift):
    rng = np.random.default_rng(32)
    B, C, L, K = 3, 3, 700, 90
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(42, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    grad_out = rng.standard_normal((B, K)).astype(np.float32)
    gw, gb = _backward(h, x, 4, grad_out, lam, shift, False)
    check_backward(x, kr, gw, gb, grad_out, None, lam, shift)
    if lam == 0.0:
        assert np.all(gw == 0) and np.all(gb == 0)


def test_shortest_series_and_single_positions():
    rng = np.random.default_rng(33)
    for (B, C, L, K) in ((2, 1, 11, 30), (1, 9, 61, 60), (3, 2, 130, 60)):
        x = rng.standard_normal((B, C, L)).astype(np.float32)
        h = rocket.rocket_make_kernels(43, K, C, L)
        kr = rocket.rocket_kernels_view_get(h)
        grad_out = rng.standard_normal((B, K)).astype(np.float32)
        gw, gb = _backward(h, x, 4, grad_out, 3.0, -3.0, False)
        check_backward(x, kr, gw, gb, grad_out, None, 3.0, -3.0)


def _few_rows(kr, L):
    """kernels that the backward pass handles as one strip over all rows: dilation of at least
    256 and at most 20 rows of d output positions (the partial last row included)"""
    d = kr["dilation"].astype(np.int64)
    n = L + 2 * kr["padding"].astype(np.int64) - (kr["length"].astype(np.int64) - 1) * d
    return (d >= 256) & (-(-n // d) <= 20)


def test_config3_full_size_sample():
    """B=60 x 20 x 50,000, K=10,000: forward max+softPPV then backward with the max
    sub-gradient, in the launch shape the benchmark times; the oracle checks a
    dilation-stratified sample of at least 128 kernels summed over the whole batch, at least
    eight of them large-dilation kernels with few rows."""
    import torch
    cfg = synth.CONFIGS[3]
    B, K, mask = cfg["B"], cfg["K"], cfg["features"]
    x = synth.make_input(3)
    h, kr = sampled(synth.seed_k(3), K, cfg["C"], cfg["L"])
    grad_out = synth.make_upstream_grad(3, B, 2 * K)
    print("config3 backward run", flush=True)
    xd = _gpu(x)
    gw, gb = rocket.rocket_soft_ppv_backward(h, xd, mask, _gpu(grad_out), 10.0, -3.0, True)
    torch.cuda.synchronize()
    gw, gb = gw.cpu().numpy(), gb.cpu().numpy()
    few = _few_rows(kr, cfg["L"])
    extra = np.nonzero(few)[0][:: max(1, int(few.sum()) // 12)][:12]
    sel = np.unique(np.concatenate([synth.pick_kernels(kr, 176, seed=3), extra])).astype(np.int32)
    print("config3 oracle forward on", len(sel), "kernels", flush=True)
    stable = _stable_argmax(x, kr, sel=sel)
    sel = sel[stable]
    assert len(sel) >= 128 and int(few[sel].sum()) >= 8, (len(sel), int(few[sel].sum()))
    g_soft, g_max = _split(grad_out, mask, K)
    rep = {}
    print("config3 oracle backward on", len(sel), "kernels,", int(few[sel].sum()), "with few rows", flush=True)
    check_backward(x, kr, gw, gb, g_soft, g_max, 10.0, -3.0, sel=sel, report=rep)
    print("config3 worst error / bound:", rep["worst_ratio"], flush=True)
    # without the max plane
    gw2, gb2 = rocket.rocket_soft_ppv_backward(h, xd, mask, _gpu(grad_out), 10.0, -3.0, False)
    torch.cuda.synchronize()
    check_backward(x, kr, gw2.cpu().numpy(), gb2.cpu().numpy(), g_soft, None, 10.0, -3.0, sel=sel[::4])


def test_backward_is_repeatable_and_overwrites():
    import torch
    rng = np.random.default_rng(34)
    B, C, L, K = 2, 4, 900, 64
    x = _gpu(rng.standard_normal((B, C, L)).astype(np.float32))
    h = rocket.rocket_make_kernels(44, K, C, L)
    v = rocket.rocket_kernels_view_get(h)
    g = _gpu(rng.standard_normal((B, K)).astype(np.float32))
    gw = torch.full((len(v["weights"]),), float("nan"), device="cuda")
    gb = torch.full((K,), float("nan"), device="cuda")
    rocket.rocket_soft_ppv_backward(h, x, 4, g, grad_w=gw, grad_b=gb)
    torch.cuda.synchronize()
    a, b = gw.cpu().numpy().copy(), gb.cpu().numpy().copy()
    assert np.all(np.isfinite(a)) and np.all(np.isfinite(b))
    rocket.rocket_soft_ppv_backward(h, x, 4, g, grad_w=gw, grad_b=gb)
    torch.cuda.synchronize()
    # every sum is taken in a fixed order without atomics: the bits repeat
    assert np.array_equal(gw.cpu().numpy(), a)
    assert np.array_equal(gb.cpu().numpy(), b)


def test_batch_that_uses_the_per_xcd_mapping():
    """8 series of more than 8,192 samples: the launch maps series to XCDs; all planes, max included"""
    rng = np.random.default_rng(77)
    B, C, L, K = 8, 2, 9001, 48
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(3, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    grad_out = rng.standard_normal((B, 3 * K)).astype(np.float32)
    print("backward, per-XCD mapping", flush=True)
    gw, gb = _backward(h, x, 7, grad_out, 10.0, -3.0, True)
    g_soft, g_max = _split(grad_out, 7, K)
    sel = np.nonzero(_stable_argmax(x, kr))[0].astype(np.int32)
    assert len(sel) > K // 2
    check_backward(x, kr, gw, gb, g_soft, g_max, 10.0, -3.0, sel=sel)


def _extreme_kernels(L, C, rng):
    """Hand-built kernels that between them reach every code path of the backward kernel: every
    length at the dilations around each path switch (1..17 LDS-staged / register strips, 63..65,
    255..257 where a lane starts taking several column blocks, a third of the largest, the largest
    and its neighbour), padded and not; and, per length, kernels whose outputs form exactly 1, 2,
    8, 9, 20, 21, 24 and 25 rows of d positions at a dilation of 256 or more (the one-strip path
    holds 8 or 20 rows; 21 and more fall back to bands of 16 + 4 + 1 and 16 + 8 + 1 rows) and 31,
    47 and 63 rows at smaller dilations (bands of 32 rows followed by every remainder height)."""
    specs = []
    for ln in (7, 9, 11):
        dmax = (L - 1) // (ln - 1)
        ds = set(range(1, 18)) | {63, 64, 65, 100, 255, 256, 257, dmax // 3, dmax - 1, dmax}
        for d in sorted(d for d in ds if 1 <= d <= dmax):
            for padded in (False, True):
                specs.append((ln, d, padded))
        for want_rows, dmin, dtop in [(r, 256, dmax) for r in (1, 2, 8, 9, 20, 21, 24, 25)] + \
                                     [(r, 16, 255) for r in (31, 47, 63)]:
            found = 0
            for d in range(dmin, dtop + 1):
                for padded in (False, True):
                    n = L + ((ln - 1) * d // 2 * 2 if padded else 0) - (ln - 1) * d
                    if n >= 1 and -(-n // d) == want_rows and found < 2:
                        specs.append((ln, d, padded))
                        found += 1
    length = np.array([s[0] for s in specs], np.int32)
    dil = np.array([s[1] for s in specs], np.int32)
    pad = np.array([(s[0] - 1) * s[1] // 2 if s[2] else 0 for s in specs], np.int32)
    nch = rng.integers(1, min(C, 9) + 1, len(specs)).astype(np.int32)
    nch[::7] = 1
    chans = np.concatenate([rng.permutation(C)[:m] for m in nch]).astype(np.int32)
    w = rng.standard_normal(int((nch * length).sum())).astype(np.float32)
    bias = rng.uniform(-1, 1, len(specs)).astype(np.float32)
    return length, dil, pad, bias, nch, chans, w


@pytest.mark.parametrize("L", [2000, 9000])
@pytest.mark.parametrize("u8", [False, True])
def test_imported_extreme_kernels(L, u8):
    """the backward twin of the forward test of the same name: every kernel of _extreme_kernels,
    softPPV alone on every kernel and with the max sub-gradient on those with a clear arg-max,
    float32 and 8-bit input"""
    import torch
    rng = np.random.default_rng(50 + L)
    C, B = 9, 3
    length, dil, pad, bias, nch, chans, w = _extreme_kernels(L, C, rng)
    K = len(length)
    h = rocket.rocket_kernels_import(K, C, L, length, dil, pad, bias, nch, chans, w)
    kr = rocket.rocket_kernels_view_get(h)
    assert np.array_equal(kr["dilation"], dil) and np.array_equal(kr["weights"], w)
    n = L + 2 * pad.astype(np.int64) - (length - 1) * dil.astype(np.int64)
    nrows = -(-n // dil)
    big = dil >= 256
    for r in (1, 2, 8, 9, 20, 21, 24, 25):
        assert np.any(big & (nrows == r)) or L < 9000, r
    if u8:
        raw = rng.integers(0, 256, size=(B, C, L)).astype(np.uint8)
        x = oracle.znormalize_u8(raw)
        xd = _gpu(raw)
        entry = rocket.rocket_soft_ppv_backward_u8
    else:
        x = rng.standard_normal((B, C, L)).astype(np.float32)
        xd = _gpu(x)
        entry = rocket.rocket_soft_ppv_backward
    lam, shift = 4.0, -3.0
    g = rng.standard_normal((B, 2 * K)).astype(np.float32)
    print("backward extreme kernels", L, u8, K, "soft only", flush=True)
    gw, gb = entry(h, xd, 4, _gpu(np.ascontiguousarray(g[:, K:])), lam, shift, False)
    torch.cuda.synchronize()
    rep = {}
    check_backward(x, kr, gw.cpu().numpy(), gb.cpu().numpy(), g[:, K:], None, lam, shift, report=rep)
    print("worst error / bound:", rep["worst_ratio"], flush=True)
    print("backward extreme kernels", L, u8, K, "with max", flush=True)
    gw, gb = entry(h, xd, 5, _gpu(g), lam, shift, True)
    torch.cuda.synchronize()
    sel = np.nonzero(_stable_argmax(x, kr))[0].astype(np.int32)
    assert len(sel) > K // 2
    check_backward(x, kr, gw.cpu().numpy(), gb.cpu().numpy(), g[:, K:], g[:, :K], lam, shift, sel=sel, report=rep)
    print("worst error / bound:", rep["worst_ratio"], flush=True)


def test_exact_ties_send_the_max_gradient_to_the_first_position():
    """Small-integer samples through kernels with one non-zero tap per channel: every sum is exact
    in float32 and in float64, the largest output is attained at many positions with different
    windows, and the sub-gradient of the max must come from the first of them (the paper's max
    pooling has no tie rule; first position is this build's reading, and the oracle's).  Dilations
    on both sides of 256, where a lane meets its positions out of order."""
    import torch
    rng = np.random.default_rng(61)
    C, B, L = 3, 2, 9000
    specs = []
    for ln in (7, 9, 11):
        dmax = (L - 1) // (ln - 1)
        for d in (1, 5, 40, 200, 257, 300, 431, 600, dmax // 2, dmax):
            for padded in (False, True):
                specs.append((ln, d, padded))
    K = len(specs)
    length = np.array([s[0] for s in specs], np.int32)
    dil = np.array([s[1] for s in specs], np.int32)
    pad = np.array([(s[0] - 1) * s[1] // 2 if s[2] else 0 for s in specs], np.int32)
    nch = rng.integers(1, C + 1, K).astype(np.int32)
    chans = np.concatenate([rng.permutation(C)[:m] for m in nch]).astype(np.int32)
    rows = []
    for k in range(K):
        for _ in range(nch[k]):
            row = np.zeros(length[k], np.float32)
            row[rng.integers(0, length[k])] = float(rng.choice([1.0, 2.0, -1.0]))
            rows.append(row)
    w = np.concatenate(rows)
    bias = rng.integers(-2, 3, K).astype(np.float32) * 0.25
    h = rocket.rocket_kernels_import(K, C, L, length, dil, pad, bias, nch, chans, w)
    kr = rocket.rocket_kernels_view_get(h)
    x = rng.integers(-2, 3, size=(B, C, L)).astype(np.float32)
    o = oracle.transform(x, kr)
    assert np.mean(o["gap"] == 0.0) > 0.9          # ties nearly everywhere
    g = np.zeros((B, 2 * K), np.float32)
    g[:, :K] = rng.integers(1, 4, size=(B, K)).astype(np.float32)     # max plane only: integer gradients
    print("backward exact ties", flush=True)
    gw, gb = rocket.rocket_soft_ppv_backward(h, _gpu(x), 5, _gpu(g), 10.0, -3.0, True)
    torch.cuda.synchronize()
    gw_ref, gb_ref = oracle.backward(x, kr, g[:, K:].astype(np.float64), g[:, :K].astype(np.float64), lam=10.0, shift=-3.0)
    # all quantities are small integers (the soft plane's upstream gradient is zero): exact equality
    assert np.array_equal(gw.cpu().numpy().astype(np.float64), gw_ref)
    assert np.array_equal(gb.cpu().numpy().astype(np.float64), gb_ref)
