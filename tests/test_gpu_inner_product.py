"""GPU parity of hgc_inner_product_forward against the FP64 oracle, through the C ABI.

Tolerance as for the convolution: |gpu - oracle| <= 4e-3 * sum|w*x| + 1e-3; integer-valued inputs
whose partial sums stay below 2048 must match exactly.
"""
import numpy as np
import pytest

import paper_1901_00858_amd as hgc
from workloads import uniform01, normal01

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def tensors(N, K, M, seed):
    """x ~ U[-1,1], w ~ N(0, 2/K) (He), b ~ U[-0.1,0.1], from the counter-based generator."""
    x = (2.0 * uniform01(seed, 0, N * K) - 1.0).astype(np.float16).reshape(N, K)
    w = (normal01(seed, 1, M * K) * np.sqrt(2.0 / K)).astype(np.float16).reshape(M, K)
    b = (0.2 * uniform01(seed, 2, M) - 0.1).astype(np.float16)
    return x, w, b


def run(desc, x, w, b, offset=0):
    """One call; offset shifts every base pointer by that many halves (alignment cases)."""
    import torch

    def dev(a):
        if a is None:
            return None
        flat = torch.empty(a.size + offset, dtype=torch.float16, device="cuda")
        flat[offset:].copy_(torch.from_numpy(np.ascontiguousarray(a).reshape(-1)))
        return flat[offset:]
    xd, wd, bd = dev(x), dev(w), dev(b)
    N, K, M = desc[0], desc[1], desc[2]
    ybuf = torch.empty(N * M + offset, dtype=torch.float16, device="cuda")
    ybuf.view(torch.int16).fill_(0x7E00)                      # NaN pattern: unwritten outputs show up
    y = ybuf[offset:]
    d = hgc.InnerProductDesc.make(desc)
    st = hgc.inner_product_forward_raw(d, xd.data_ptr(), wd.data_ptr(), bd.data_ptr() if bd is not None else 0,
                                       y.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == 0, hgc.status_string(st)
    torch.cuda.synchronize()
    return y.cpu().numpy().reshape(N, M)


def check(oracle, desc, x, w, b, y, tag):
    pre, mag = oracle.inner_product_forward(desc, x, w, b)
    ok, ratio, where = oracle.check(y, pre, mag, desc[4])
    assert ok, f"{tag} {desc}: |err|/bound = {ratio:.3g} at {where}: got {y[where]}, pre {pre[where]}"
    return ratio


SHAPES = [
    # N, K, M: ragged everything (element-load path), then the vector path with tails in M and N
    (1, 1, 1), (3, 37, 5), (2, 40, 7), (5, 1000, 33), (1, 512, 64), (2, 520, 130), (4, 4096, 100),
    (7, 1024, 257), (8, 2048, 64), (9, 520, 130), (16, 256, 40), (17, 64, 3000), (64, 1024, 100),
    # more than eight images (matrix-core path): K below, at and past a 128-value block, ragged rows and images,
    # one, two and three passes of 32 images
    (10, 8, 1), (12, 136, 17), (32, 128, 16), (33, 1032, 50), (70, 392, 33), (16, 4096, 256),
    # four to eight images take that path on long layers only
    (4, 72, 2048), (5, 264, 2100), (8, 64, 2047),
]


@pytest.mark.parametrize("shape", SHAPES, ids=[f"{n}x{k}x{m}" for n, k, m in SHAPES])
def test_shapes(oracle, shape):
    N, K, M = shape
    x, w, b = tensors(N, K, M, seed=N + K + M)
    for bias, relu in ((1, 0), (1, 1), (0, 1)):
        desc = (N, K, M, bias, relu)
        say(f"[ip] {desc}")
        y = run(desc, x, w, b if bias else None)
        check(oracle, desc, x, w, b if bias else None, y, "ip")


def test_unaligned_bases_take_the_element_path(oracle):
    for shape in [(2, 512, 40), (3, 264, 9)]:
        N, K, M = shape
        x, w, b = tensors(N, K, M, seed=5)
        desc = (N, K, M, 1, 1)
        for off in (1, 3, 4, 8):
            say(f"[ip unaligned] {desc} offset {off} halves")
            y = run(desc, x, w, b, offset=off)
            check(oracle, desc, x, w, b, y, f"offset {off}")


def test_integer_inputs_are_exact(oracle):
    rng = np.random.default_rng(3)
    for N, K, M in [(1, 128, 10), (4, 96, 70), (8, 100, 5)]:
        x = rng.integers(-4, 5, size=(N, K)).astype(np.float16)
        w = rng.integers(-2, 3, size=(M, K)).astype(np.float16)
        b = rng.integers(-8, 9, size=(M,)).astype(np.float16)
        desc = (N, K, M, 1, 0)
        pre, _ = oracle.inner_product_forward(desc, x, w, b)
        say(f"[ip int] {desc}")
        y = run(desc, x, w, b)
        assert np.array_equal(y.astype(np.float64), pre), desc


FC = [("alexnet fc6", 9216, 4096), ("vgg16 fc6", 25088, 4096), ("fc7", 4096, 4096), ("fc8", 4096, 1000)]


@pytest.mark.parametrize("name,K,M", FC, ids=[f[0].replace(" ", "_") for f in FC])
def test_classifier_layers_at_full_size(oracle, name, K, M):
    """The fully connected layers of the AlexNet- and VGG-16-shaped nets, N = 1 and N = 4, every output."""
    for N in (1, 4):
        x, w, b = tensors(N, K, M, seed=K + M)
        desc = (N, K, M, 1, 1)
        say(f"[ip full] {name} {desc}")
        y = run(desc, x, w, b)
        check(oracle, desc, x, w, b, y, name)


def test_a_conv_tensor_is_accepted_as_it_is(oracle):
    """x given as [N][C][H][W]: the layer equals a convolution whose kernel covers the image."""
    import torch
    N, C, H, W, M = 2, 16, 7, 7, 24
    x, w, b = tensors(N, C * H * W, M, seed=11)
    x4 = torch.from_numpy(x.reshape(N, C, H, W)).cuda()
    y = hgc.inner_product_forward((N, C * H * W, M, 1, 0), x4, torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda())
    torch.cuda.synchronize()
    pre, mag = oracle.conv2d_forward((N, C, H, W, M, H, 1, 0, 1, 1, 0), x.reshape(N, C, H, W), w.reshape(M, C, H, W), b)
    ok, ratio, where = oracle.check(y.cpu().numpy(), pre.reshape(N, M), mag.reshape(N, M), 0)
    assert ok, (ratio, where)
