"""Shared plumbing of the GPU parity tests: run a layer through the C ABI and
compare with the oracle under the stated tolerance."""
import sys

import numpy as np

import paper_1901_00858_amd as hgc
from workloads import make_tensors


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def to_dev(a):
    import torch
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_layer(L, x, w, b, use_ws=False, poison=True, packed=False):
    """One call through hgc_conv2d_forward(_ws|_packed). Returns y as a numpy float16 array."""
    import torch
    xd, wd, bd = to_dev(x), to_dev(w), to_dev(b)
    y = torch.empty(L.y_shape, dtype=torch.float16, device="cuda")
    if poison:
        y.view(torch.int16).fill_(0x7E00)          # NaN bit pattern: unwritten outputs show up
    if packed:
        wp = torch.empty(hgc.conv2d_packed_weights_size(L), dtype=torch.uint8, device="cuda")
        wp.fill_(0x7E)                              # every byte is overwritten by the pack kernel
        hgc.conv2d_pack_weights(L, wd, wp)
        need = hgc.conv2d_workspace_size(L)
        ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        hgc.conv2d_forward_packed(L, xd, wp, bd, y, ws)
    elif use_ws:
        need = hgc.conv2d_workspace_size(L)
        ws = None
        if need:
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            ws.fill_(0xFF)                          # NaN pattern for FP32 partial sums
        hgc.conv2d_forward_ws(L, xd, wd, bd, y, ws)
    else:
        hgc.conv2d_forward(L, xd, wd, bd, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def assert_full(oracle, L, x, w, b, y, tag=""):
    pre, mag = oracle.conv2d_forward(L.desc(), x, w, b)
    ok, ratio, where = oracle.check(y, pre, mag, L.relu)
    assert ok, f"{tag} {L}: |err|/bound = {ratio:.3g} at {where}: got {y[where]}, pre {pre[where]}"
    return ratio


def sample_points(L, rng, count):
    """Corners, edges, first/last image and channel, plus random coordinates."""
    pts = []
    for n in {0, L.N - 1}:
        for m in {0, L.M - 1, L.M // 2}:
            for oh in {0, L.Ho - 1, L.Ho // 2}:
                for ow in {0, L.Wo - 1, L.Wo // 2}:
                    pts.append((n, m, oh, ow))
    r = np.stack([rng.integers(0, d, count) for d in L.y_shape], axis=1)
    return np.concatenate([np.array(pts, dtype=np.int64), r], axis=0)


def assert_points(oracle, L, x, w, b, y, idx, tag=""):
    pre, mag = oracle.conv2d_points(L.desc(), x, w, b, idx)
    got = y[tuple(idx.T)]
    ok, ratio, where = oracle.check(got, pre, mag, L.relu)
    assert ok, f"{tag} {L}: |err|/bound = {ratio:.3g} at {idx[where[0]]}"
    return ratio
