"""GPU parity of hgc_max_pool_forward against the oracle, through the C ABI: exact.

The result of a maximum is one of the inputs, so every output must equal the oracle's as a number
(+0 and -0 compare equal; the inputs hold no NaN).
"""
import numpy as np
import pytest

import paper_1901_00858_amd as hgc
from workloads import normal01

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def values(shape, seed):
    return normal01(seed, 0, int(np.prod(shape))).astype(np.float16).reshape(shape)


def run(desc, x, offset=0):
    import torch
    d = hgc.MaxPoolDesc.make(desc)
    st, ho, wo = hgc.max_pool_output_size_raw(d)
    assert st == 0
    xbuf = torch.empty(x.size + offset, dtype=torch.float16, device="cuda")
    xd = xbuf[offset:]
    xd.copy_(torch.from_numpy(np.ascontiguousarray(x).reshape(-1)))
    n = d.N * d.C * ho * wo
    ybuf = torch.empty(n + offset, dtype=torch.float16, device="cuda")
    ybuf.view(torch.int16).fill_(0x7E00)                       # NaN pattern: unwritten outputs show up
    yd = ybuf[offset:]
    st = hgc.max_pool_forward_raw(d, xd.data_ptr(), yd.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == 0, hgc.status_string(st)
    torch.cuda.synchronize()
    return yd.cpu().numpy().reshape(d.N, d.C, ho, wo)


def check(oracle, desc, x, y, tag):
    ref = oracle.max_pool_forward(desc, x)
    assert y.shape == ref.shape, f"{tag} {desc}: shape {y.shape} vs {ref.shape}"
    bad = np.argwhere(~(y.astype(np.float32) == ref.astype(np.float32)))
    assert bad.size == 0, f"{tag} {desc}: {len(bad)} differ, first at {tuple(bad[0])}: got {y[tuple(bad[0])]}, want {ref[tuple(bad[0])]}"


WINDOWS = [(2, 2, 0), (3, 2, 0), (3, 2, 1), (3, 1, 1), (2, 2, 1), (3, 3, 0), (5, 2, 2), (1, 1, 0), (2, 1, 0), (4, 3, 1)]
SHAPES = [(1, 1, 5, 5), (2, 3, 7, 9), (1, 2, 12, 6), (2, 5, 13, 13), (3, 4, 16, 16), (1, 7, 15, 24), (2, 3, 28, 28)]


@pytest.mark.parametrize("shape", SHAPES, ids=["x".join(map(str, s)) for s in SHAPES])
def test_windows(oracle, shape):
    x = values(shape, seed=sum(shape))
    for k, s, p in WINDOWS:
        if shape[2] + 2 * p < k or shape[3] + 2 * p < k:
            continue
        desc = shape + (k, s, p)
        say(f"[pool] {desc}")
        check(oracle, desc, x, run(desc, x), "pool")


def test_vector_form_and_its_edges(oracle):
    """2x2 / 2 with rows that are a multiple of 8: even and odd heights, one vector a row, unaligned bases."""
    for shape in [(2, 3, 8, 8), (1, 5, 9, 16), (2, 2, 7, 24), (3, 64, 56, 56), (1, 3, 2, 8), (1, 3, 3, 8), (2, 2, 14, 14)]:
        x = values(shape, seed=7)
        desc = shape + (2, 2, 0)
        say(f"[pool-2x2] {desc}")
        check(oracle, desc, x, run(desc, x), "2x2")
        for off in (1, 4):
            check(oracle, desc, x, run(desc, x, offset=off), f"2x2 offset {off}")


def test_signed_zeros_and_negative_images(oracle):
    x = -np.abs(values((1, 2, 6, 8), seed=3)) - np.float16(0.5)
    for desc in [(1, 2, 6, 8, 3, 2, 1), (1, 2, 6, 8, 2, 2, 0)]:
        y = run(desc, x)
        check(oracle, desc, x, y, "negative")
        assert np.all(y < 0)                                   # padding is no candidate
    z = np.zeros((1, 1, 4, 8), dtype=np.float16)
    z[0, 0, ::2, ::2] = -0.0
    check(oracle, (1, 1, 4, 8, 2, 2, 0), z, run((1, 1, 4, 8, 2, 2, 0), z), "zeros")


def test_benchmark_size(oracle):
    """VGG-16's first pooling at the batch the benchmark's larger runs use: 16 x 64 x 224 x 224."""
    shape = (16, 64, 224, 224)
    x = values(shape, seed=11)
    desc = shape + (2, 2, 0)
    say(f"[pool-full] {desc}")
    check(oracle, desc, x, run(desc, x), "full")


def test_binding_wrapper(oracle):
    import torch
    x = values((2, 4, 10, 10), seed=5)
    y = hgc.max_pool_forward((2, 4, 10, 10, 3, 2, 0), torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    check(oracle, (2, 4, 10, 10, 3, 2, 0), x, y.cpu().numpy(), "wrapper")
    assert hgc.max_pool_output_size((1, 96, 55, 55, 3, 2, 0)) == (27, 27)
