"""GPU parity on randomly drawn problem shapes: channel counts, series lengths around the
kernels' internal boundaries (64, 256, 4096, 8192 samples), kernel counts, batch sizes, feature
masks, lambda and shift, float32 or 8-bit input; forward always, backward when softPPV is in
the mask.  Every case is seeded by its index.  Needs an MI355X."""
import numpy as np
import pytest

import oracle
from paper_2301_08527_amd import rocket
from parity import check_backward, check_forward

pytestmark = pytest.mark.gpu

CASES = 48


def _case(i):
    rng = np.random.default_rng([20230120, i])
    p = dict(
        C=int(rng.choice([1, 2, 3, 5, 9, 12, 20])),
        L=int(rng.choice([11, 12, 50, 64, 255, 256, 257, 1000, 4097, 8192, 8193, 20000, 65536, 100001])),
        K=int(rng.integers(1, 200)), B=int(rng.integers(1, 5)), mask=int(rng.integers(1, 8)),
        lam=float(rng.choice([0.5, 3.0, 10.0])), shift=float(rng.choice([-3.0, 3.0, 0.0])),
        seed=int(rng.integers(0, 1 << 30)), u8=bool(rng.random() < 0.3), scale=float(rng.choice([0.1, 1.0])))
    return p, rng


def test_random_shapes():
    import torch
    for i in range(CASES):
        p, rng = _case(i)
        print("case", i, p, flush=True)
        B, C, L, K, mask, lam, shift = p["B"], p["C"], p["L"], p["K"], p["mask"], p["lam"], p["shift"]
        h = rocket.rocket_make_kernels(p["seed"], K, C, L)
        kr = rocket.rocket_kernels_view_get(h)
        if p["u8"]:
            raw = rng.integers(0, 256, size=(B, C, L)).astype(np.uint8)
            x = oracle.znormalize_u8(raw)
            out = rocket.rocket_transform_u8(h, torch.from_numpy(raw).cuda(), mask, lam, shift)
        else:
            x = (rng.standard_normal((B, C, L)) * p["scale"]).astype(np.float32)
            out = rocket.rocket_transform(h, torch.from_numpy(x).cuda(), mask, lam, shift)
        torch.cuda.synchronize()
        check_forward(x, kr, out.cpu().numpy(), mask, lam, shift)
        if mask & 4 and L * K * B * C < 3e7:
            F = bin(mask).count("1")
            g = rng.standard_normal((B, F * K)).astype(np.float32)
            inc = bool(mask & 1) and rng.random() < 0.5
            gw, gb = rocket.rocket_soft_ppv_backward(h, torch.from_numpy(x).cuda(), mask, torch.from_numpy(g).cuda(),
                                                     lam, shift, inc)
            torch.cuda.synchronize()
            sel = None
            if inc:     # the max sub-gradient is compared where fp32 and fp64 agree on the arg-max
                o = oracle.transform(x, kr, lam=lam, shift=shift)
                sel = np.nonzero(o["gap"].min(axis=0) > 1e-3)[0].astype(np.int32)
            if sel is None or len(sel):
                check_backward(x, kr, gw.cpu().numpy(), gb.cpu().numpy(), g[:, (F - 1) * K:],
                               g[:, :K] if inc else None, lam, shift, sel=sel)
        h.free()
