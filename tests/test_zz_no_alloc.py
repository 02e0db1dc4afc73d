"""The entry point that allocates nothing (kfac_update_factors_static: scratch in the library's static device
array) against kfac_update_factors on the same inputs: two calls in a row, the second with a smaller input,
then an input whose split plan does not fit the array."""
import numpy as np
import pytest
import torch

from paper_2007_00784_amd import kfac as K
from gpu_util import Ctx, relfro

pytestmark = pytest.mark.gpu


def _inputs(dev, N, d, T, seed, bf16=False):
    g = torch.Generator(device="cpu").manual_seed(seed)
    x = torch.relu(torch.randn((N, d, T), generator=g, dtype=torch.float32))
    x = x.to(torch.bfloat16) if bf16 else x
    return x.to(dev)


def test_static_scratch_entry_point_matches_workspace_entry_point():
    ctx = Ctx(256 << 20)
    try:
        assert K.kfac_static_scratch_bytes() == 48 << 20
        # (N, d, T, ones, decay, bf16): the first needs split partials (nsplit > 1), the second is smaller
        cases = [(64, 288, 196, 1, 0.0, False), (16, 100, 49, 1, 0.95, False), (32, 130, 64, 0, 0.5, True)]
        for k, (N, d, T, ones, decay, bf16) in enumerate(cases):
            X = _inputs(ctx.dev, N, d, T, seed=k, bf16=bf16)
            D = d + ones
            F0 = torch.randn((D, D), dtype=torch.float32, device=ctx.dev)
            F0 = F0 @ F0.T
            Fa, Fb = F0.clone(), F0.clone()
            scale = 1.0 / (N * T)
            K.kfac_update_factors(ctx.h, X, K.KFAC_LAYOUT_NDT, N, d, T, ones, scale, decay, Fa)
            K.kfac_update_factors_static(ctx.h, X, K.KFAC_LAYOUT_NDT, N, d, T, ones, scale, decay, Fb)
            torch.cuda.synchronize()
            a, b = Fa.cpu().numpy(), Fb.cpu().numpy()
            assert np.isfinite(b).all()
            assert relfro(b, a) <= 1e-4, (k, relfro(b, a))
            assert np.array_equal(a, b), k          # same kernels, same split plan: the same bits
        # a plan that needs more partial tiles than the static array holds is refused before anything is launched
        N, d, T = 32, 2304, 196
        it = dict(X=None, dtype=K.KFAC_F32, layout=K.KFAC_LAYOUT_NDT, N=N, d=d, T=T, append_ones=1, scale=1.0, decay=0.0, F=None)
        assert K.kfac_update_factors_workspace_bytes([it]) > K.kfac_static_scratch_bytes()
        X = torch.zeros((N, d, T), dtype=torch.float32, device=ctx.dev)
        F = torch.zeros((d + 1, d + 1), dtype=torch.float32, device=ctx.dev)
        with pytest.raises(K.KfacError) as e:
            K.kfac_update_factors_static(ctx.h, X, K.KFAC_LAYOUT_NDT, N, d, T, 1, 1.0, 0.0, F)
        assert e.value.code == K.KFAC_ESCRATCH
        assert "static" in K.kfac_strerror(K.KFAC_ESCRATCH)
    finally:
        ctx.close()
