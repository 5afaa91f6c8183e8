"""hqmq_encode_static: the encode entry point that allocates nothing (its workspace is a static array
inside the library's device image).  Its results must equal hqmq_encode's byte for byte, on two calls in
a row that share the array, the second on a smaller input."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import paper_2605_27646_amd as hq
import workloads
from gpu_util import gpu_encode

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _encode_static(x_dev, sec_dev, b_r, Cmul):
    params = hq.params_for(x_dev, sec_dev.shape[1], b_r, Cmul)
    bufs = hq.alloc_encoded(params, x_dev.device)
    for t in (bufs.codes, bufs.flags, bufs.row_off, bufs.n_outliers, bufs.status):
        t.fill_(-1)
    bufs.sigma.fill_(float("nan"))
    hq.hqmq_encode_static(params, x_dev, sec_dev, bufs)
    return bufs


def _same(bufs, want):
    torch.cuda.synchronize()
    total = int(want.n_out[-1])
    assert np.array_equal(bufs.n_outliers.cpu().numpy().view(np.uint32), want.n_out)
    assert int(bufs.status.item()) == want.status == 0
    assert np.array_equal(bufs.flags.cpu().numpy().view(np.uint32), want.flags)
    assert np.array_equal(bufs.row_off.cpu().numpy().view(np.uint32), want.row_off)
    assert np.array_equal(bufs.sigma.cpu().numpy().view(np.uint16), want.sigma)
    assert np.array_equal(bufs.codes.cpu().numpy().view(np.uint32), want.codes)
    assert np.array_equal(bufs.outliers[:total].cpu().numpy().view(np.uint16).reshape(total, 4), want.outliers)
    return total


def test_static_workspace_encode_equals_hqmq_encode():
    hq.hqmq_init()
    # first call: 8 heads, S = 256 (the headline shape's tables), ragged length; second call: a smaller
    # tensor with fewer heads, another codebook size and another head dimension, on the array the first
    # call left behind
    cases = [(1, 8, 1500, 128, 256, 6, 3.0, 0.5), (2, 3, 333, 96, 48, 4, 1.5, 1.0)]
    for (B, H, T, D, S, b_r, Cmul, sigma_g) in cases:
        wl = workloads.Workload("static", 4242 + T, 1, B, H, T, D, S, sigma_g=sigma_g)
        x = workloads.make_tensor(wl, 0, 0, "cpu").to(DEV)
        sec = hq.hqmq_build_codebooks(9, 1, H, S)[0, 0].contiguous().to(DEV)
        want = gpu_encode(x, sec, b_r, Cmul)          # hqmq_encode with a caller workspace
        assert hq.hqmq_sizes(want.params).workspace_bytes <= hq.HQMQ_STATIC_SCRATCH_BYTES
        bufs = _encode_static(x, sec, b_r, Cmul)
        assert _same(bufs, want) > 0
    # the second call again, back to back with a third on the same stream, no synchronisation between them
    a = _encode_static(x, sec, b_r, Cmul)
    b = _encode_static(x, sec, b_r, Cmul)
    _same(a, want)
    _same(b, want)


def test_static_workspace_rejects_what_does_not_fit():
    H = 64
    x = torch.zeros(1, H, 64, 128, dtype=torch.float16, device=DEV)
    sec = hq.hqmq_build_codebooks(0, 1, H, 256)[0, 0].contiguous().to(DEV)
    params = hq.params_for(x, 256)
    assert hq.hqmq_sizes(params).workspace_bytes > hq.HQMQ_STATIC_SCRATCH_BYTES
    bufs = hq.alloc_encoded(params, DEV)
    with pytest.raises(hq.HqmqError) as ei:
        hq.hqmq_encode_static(params, x, sec, bufs)
    assert ei.value.code == -3
