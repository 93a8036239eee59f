"""A chained forward pass on the GPU (convolution -> convolution -> pooling -> ... -> inner product), every
layer reading the previous layer's FP16 output, against the same chain of oracles.

The oracle chain runs on its own intermediates (each reference output rounded to FP16 is the next
layer's input); nothing the GPU produced enters it.  The two chains drift apart by what each layer's
tolerance allows, so the comparison carries a bound E on |x_gpu - x_oracle| from layer to layer:
  convolution / inner product: E_out = P + 4e-3 (mag + P) + 1e-3 + 2^-11 |ref| + 6e-8,  P = sum |w| E_in
      (P: the drift carried through the layer; 4e-3 (mag + P) + 1e-3: the layer's own tolerance on the
      GPU's input, whose sum |w x| is at most mag + P; the last terms: the oracle chain's rounding of ref)
  ReLU: unchanged (1-Lipschitz);  max pooling: E_out = the window's maximum of E_in.
Every layer's output must agree within E.  E is a worst-case bound (every deviation of a layer's inputs
is taken to pull the same way through |w|), so it grows by about sum |w| per layer and says little by the
end of the chain; beside it the test therefore holds the chains to what the arithmetic gives on average:
one FP16 rounding per layer, 2^-11 relative, so after L layers the root-mean-square difference stays
below 1e-3 of the outputs' root mean square (measured: 2 to 3e-4 at every layer).
"""
import numpy as np
import pytest

import paper_1901_00858_amd as hgc
from workloads import uniform01, normal01

pytestmark = pytest.mark.gpu


def _conv_w(M, Cg, k, seed):
    w = (normal01(seed, 1, M * Cg * k * k) * np.sqrt(2.0 / (Cg * k * k))).astype(np.float16).reshape(M, Cg, k, k)
    b = (0.2 * uniform01(seed, 2, M) - 0.1).astype(np.float16)
    return w, b


def _chain(N, C, H, W):
    """(kind, parameters) list of a small VGG-shaped net."""
    return [
        ("conv", dict(M=8, k=3, s=1, p=1, G=1, relu=1)),
        ("conv", dict(M=8, k=3, s=1, p=1, G=1, relu=1)),
        ("pool", dict(k=2, s=2, p=0)),
        ("conv", dict(M=16, k=3, s=1, p=1, G=2, relu=1)),
        ("pool", dict(k=3, s=2, p=0)),
        ("fc", dict(M=32, relu=1)),
        ("fc", dict(M=10, relu=0)),
    ]


@pytest.mark.parametrize("shape", [(2, 3, 16, 16), (1, 4, 21, 13)], ids=["2x3x16x16", "1x4x21x13"])
def test_chained_forward_pass(oracle, shape):
    import torch
    N, C, H, W = shape
    x0 = (2.0 * uniform01(1, 0, N * C * H * W) - 1.0).astype(np.float16).reshape(N, C, H, W)
    xg = torch.from_numpy(x0).cuda()                       # the GPU chain's current tensor
    xo = x0.copy()                                         # the oracle chain's current tensor (FP16)
    E = np.zeros(x0.shape, dtype=np.float64)
    ref = None
    for li, (kind, p) in enumerate(_chain(N, C, H, W)):
        if kind == "conv":
            c, h, w_ = xo.shape[1:]
            wt, b = _conv_w(p["M"], c // p["G"], p["k"], seed=10 + li)
            desc = (N, c, h, w_, p["M"], p["k"], p["s"], p["p"], p["G"], 1, p["relu"])
            ws = torch.empty(max(1, hgc.conv2d_workspace_size(desc)), dtype=torch.uint8, device="cuda")
            xg = hgc.conv2d_forward_ws(desc, xg, torch.from_numpy(wt).cuda(), torch.from_numpy(b).cuda(), None, ws)
            pre, mag = oracle.conv2d_forward(desc, xo, wt, b)
            P = torch.nn.functional.conv2d(torch.from_numpy(E), torch.from_numpy(np.abs(wt.astype(np.float64))),
                                           stride=p["s"], padding=p["p"], groups=p["G"]).numpy()
            ref = np.maximum(pre, 0.0) if p["relu"] else pre
            E = P + 4e-3 * (mag + P) + 1e-3 + 2.0 ** -11 * np.abs(ref) + 6e-8
            xo = ref.astype(np.float16)
        elif kind == "pool":
            c, h, w_ = xo.shape[1:]
            desc = (N, c, h, w_, p["k"], p["s"], p["p"])
            xg = hgc.max_pool_forward(desc, xg)
            xo = oracle.max_pool_forward(desc, xo)
            E = torch.nn.functional.max_pool2d(torch.from_numpy(E), p["k"], p["s"], p["p"], ceil_mode=True).numpy()
            assert E.shape == xo.shape
            ref = xo.astype(np.float64)
        else:
            K = int(np.prod(xo.shape[1:]))
            wt = (normal01(10 + li, 1, p["M"] * K) * np.sqrt(2.0 / K)).astype(np.float16).reshape(p["M"], K)
            b = (0.2 * uniform01(10 + li, 2, p["M"]) - 0.1).astype(np.float16)
            desc = (N, K, p["M"], 1, p["relu"])
            xg = hgc.inner_product_forward(desc, xg, torch.from_numpy(wt).cuda(), torch.from_numpy(b).cuda())
            pre, mag = oracle.inner_product_forward(desc, xo.reshape(N, K), wt, b)
            P = E.reshape(N, K) @ np.abs(wt.astype(np.float64)).T
            ref = np.maximum(pre, 0.0) if p["relu"] else pre
            E = P + 4e-3 * (mag + P) + 1e-3 + 2.0 ** -11 * np.abs(ref) + 6e-8
            xo = ref.astype(np.float16)
        torch.cuda.synchronize()
        got = xg.cpu().numpy().astype(np.float64).reshape(ref.shape)
        err = np.abs(got - ref)
        worst = np.unravel_index(np.argmax(err / E), err.shape)
        rel = np.sqrt(np.mean(err ** 2)) / np.sqrt(np.mean(ref ** 2))
        print(f"[chain] layer {li} {kind}: worst |err|/E = {err[worst] / E[worst]:.3f}, median E = {np.median(E):.2e}, "
              f"rms(err)/rms(ref) = {rel:.2e}", flush=True)
        assert np.all(np.isfinite(got))
        assert np.all(err <= E), f"layer {li} ({kind}): |err| {err[worst]} > bound {E[worst]} at {worst}"
        assert rel <= 1e-3, f"layer {li} ({kind}): rms difference {rel:.3e} of the outputs' rms"
    assert ref.shape == (N, 10)
