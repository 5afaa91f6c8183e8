"""The whole path (encode, decode, fused attention) enqueues plain kernel launches only, so a caller can
record it into a HIP graph.  The graph is replayed several times with eager work in between, and every
replay must reproduce the eager bytes."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import paper_2605_27646_amd as hq
import workloads

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def test_graph_replays_match_eager():
    B, H, T, S, G = 1, 4, 700, 64, 4
    wl = workloads.Workload("graph", 900, 1, B, H, T, 128, S, sigma_g=0.8)
    k = workloads.make_tensor(wl, 0, 0, "cpu").to(DEV)
    v = workloads.make_tensor(wl, 0, 1, "cpu").to(DEV)
    cb = hq.hqmq_build_codebooks(1, 1, H, S).to(DEV)
    sec_k, sec_v = cb[0, 0].contiguous(), cb[0, 1].contiguous()
    params = hq.params_for(k, S)
    ek, ev = hq.alloc_encoded(params, DEV), hq.alloc_encoded(params, DEV)
    ws = hq.alloc_batch_workspace(params, 2, DEV)
    batch = hq.EncodeBatch(params, [k, v], [sec_k, sec_v], [ek, ev], ws)
    ok, ov = torch.empty_like(k), torch.empty_like(v)
    dec = hq.DecodeBatch(params, [ek, ev], [sec_k, sec_v], [ok, ov])
    q = torch.randn(B, H * G, 128, generator=torch.Generator().manual_seed(3)).to(torch.float16).to(DEV)
    o = torch.empty_like(q)
    aws = torch.empty(hq.hqmq_attend_workspace_bytes(params, H * G), dtype=torch.uint8, device=DEV)
    o2 = torch.empty_like(q)
    lse = torch.empty(B, H * G, dtype=torch.float32, device=DEV)
    vis = torch.randint(0, T + 1, (B, H * G), generator=torch.Generator().manual_seed(4), dtype=torch.int32).to(DEV)
    aws2 = torch.empty_like(aws)

    es = hq.alloc_encoded(params, DEV)          # K once more through the entry point that takes no workspace

    def path():
        hq.hqmq_encode_static(params, k, sec_k, es)
        hq.hqmq_encode_batch(batch)
        hq.hqmq_decode_batch(dec)
        hq.hqmq_attend(params, q, 0.09, ek, sec_k, ev, sec_v, o, aws)
        hq.hqmq_attend_masked(params, q, 0.09, ek, sec_k, ev, sec_v, vis, o2, aws2, lse)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (es.codes, es.row_off, es.n_outliers, es.status,
                                    ek.codes, ek.flags, ek.row_off, ek.n_outliers, ev.codes, ok.view(torch.int16),
                                    ov.view(torch.int16), o.view(torch.int16), o2.view(torch.int16),
                                    lse.view(torch.int32))]

    def scrub():
        for t in (ek.codes, ek.flags, ek.row_off, ev.codes, ek.n_outliers, es.codes, es.row_off, es.n_outliers, es.status):
            t.fill_(-1)
        for t in (ok, ov, o, o2, lse):
            t.fill_(float("nan"))
        ws.fill_(0x77)
        aws.fill_(0x77)
        aws2.fill_(0x77)

    hq.hqmq_init()                              # per-device set-up outside any capture
    path()
    want = snapshot()
    assert int(ek.n_outliers[-1]) > 0
    assert torch.equal(es.codes, ek.codes) and torch.equal(es.row_off, ek.row_off)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        path()                                  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        path()
    for rep in range(3):
        scrub()
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert torch.equal(a, b), rep
        # eager work of the program's own between the replays
        path()
        torch.cuda.synchronize()
