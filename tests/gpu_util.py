"""Helpers shared by the GPU parity tests: run the library through its Python binding (which
calls the C ABI) and bring the results back as numpy arrays laid out like the oracle's."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

import oracle
import paper_2605_27646_amd as hq

NEAR_TIE = 1e-6          # score gap below which two codewords count as tied (spec rule)
RECON_TOL = 1e-3         # max-abs reconstruction error relative to the chunk norm


@dataclass
class GpuEncoded:
    params: hq.HqmqParams
    bufs: hq.EncodedBuffers
    codes: np.ndarray
    sigma: np.ndarray       # uint16 bit patterns
    flags: np.ndarray       # uint32
    row_off: np.ndarray     # uint32
    n_out: np.ndarray       # uint32
    outliers: np.ndarray    # uint16 [total (clipped to capacity), 4]
    status: int


def gpu_encode(x_dev: torch.Tensor, sec_dev: torch.Tensor, b_r=6, Cmul=3.0, flags=0,
               outlier_capacity=None) -> GpuEncoded:
    S = sec_dev.shape[1]
    params = hq.params_for(x_dev, S, b_r, Cmul, flags)
    bufs = hq.alloc_encoded(params, x_dev.device, outlier_capacity)
    ws = hq.alloc_workspace(params, x_dev.device)
    ws.fill_(0xAB)                      # the workspace needs no initialisation
    bufs.codes.fill_(-1)
    hq.hqmq_encode(params, x_dev, sec_dev, bufs, ws)
    torch.cuda.synchronize()
    n_out = bufs.n_outliers.cpu().numpy().view(np.uint32)
    total = int(n_out[-1])
    kept = min(total, bufs.outlier_capacity)
    return GpuEncoded(
        params, bufs,
        bufs.codes.cpu().numpy().view(np.uint32),
        bufs.sigma.cpu().numpy().view(np.uint16),
        bufs.flags.cpu().numpy().view(np.uint32),
        bufs.row_off.cpu().numpy().view(np.uint32),
        n_out,
        bufs.outliers[:kept].cpu().numpy().view(np.uint16).reshape(kept, 4),
        int(bufs.status.cpu().numpy().view(np.uint32)[0]),
    )


def gpu_decode(params, bufs, sec_dev, like: torch.Tensor) -> np.ndarray:
    out = torch.empty_like(like)
    out.fill_(float("nan"))
    hq.hqmq_decode(params, bufs, sec_dev, out)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16)


def upload_encoded(e: oracle.Encoded, device) -> hq.EncodedBuffers:
    """Device copy of an oracle-encoded tensor (decode parity on identical bytes)."""
    def i32(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int32)).to(device)
    outl = e.outliers if e.outliers.size else np.zeros((0, 4), np.uint16)
    return hq.EncodedBuffers(
        codes=i32(e.codes), sigma=torch.from_numpy(e.sigma.view(np.float16).copy()).to(device),
        flags=i32(e.flags), row_off=i32(e.row_off),
        outliers=torch.from_numpy(outl.view(np.float16).copy()).to(device).reshape(-1, 4),
        n_outliers=i32(e.n_out), status=torch.zeros(1, dtype=torch.int32, device=device))


def chunked(bits: np.ndarray, nc: int) -> np.ndarray:
    """[..., D] fp16 bit patterns -> [rows, nc, 4], a last partial chunk completed with +0."""
    D = bits.shape[-1]
    flat = bits.reshape(-1, D)
    if D != 4 * nc:
        pad = np.zeros((flat.shape[0], 4 * nc), np.uint16)
        pad[:, :D] = flat
        flat = pad
    return flat.reshape(-1, nc, 4)


def compare_encode(g: GpuEncoded, e: oracle.Encoded, x_bits: np.ndarray, sec: np.ndarray) -> dict:
    """Bit-exact parity on masks, offsets, counts, payload, scales and radius codes; codeword
    indices identical wherever the oracle's score gap is >= NEAR_TIE, and within NEAR_TIE of
    the best score otherwise.  Returns the counts for reporting."""
    assert np.array_equal(g.flags, e.flags), "outlier flag words differ"
    assert np.array_equal(g.n_out, e.n_out), "outlier counts differ"
    assert np.array_equal(g.row_off, e.row_off), "row offsets differ"
    assert g.status == 0
    assert np.array_equal(g.outliers, e.outliers), "outlier payload differs"
    assert np.array_equal(g.sigma, e.sigma), "per-row scales differ"
    rows = np.flatnonzero(e.searched)
    nc = e.r2.shape[1]
    assert g.codes.shape == e.codes.shape
    k_gpu, rq_gpu = oracle.unpack_rows(g.codes[rows], e.S, e.b_r, nc)
    ok = e.flag[rows] == 0
    # every index names a codeword (an index past 24 S could not be scored by the near-tie rule below)
    assert (k_gpu < 24 * e.S).all(), "codeword index outside the joint codebook"
    # flagged chunks carry code 0
    assert (k_gpu[~ok] == 0).all() and (rq_gpu[~ok] == 0).all()
    assert np.array_equal(rq_gpu[ok], e.rq[rows][ok]), "radius codes differ"
    k_or = e.k[rows]
    gap = (e.best - e.second)[rows]
    diff = ok & (k_gpu != k_or)
    assert not (diff & (gap >= NEAR_TIE)).any(), "codeword index differs where the gap is >= 1e-6"
    # near ties: the GPU's pick must score within NEAR_TIE of the oracle's best
    rr, cc = np.nonzero(diff)
    chunks = chunked(x_bits, nc)
    H, T = e.H, e.T
    for r, c in zip(rr, cc):
        row = rows[r]
        h = (row // T) % H
        sc = oracle.score(chunks[row, c], sec[h], int(k_gpu[r, c]))
        assert sc >= e.best[row, c] - NEAR_TIE, (row, c, sc, e.best[row, c])
    # where the indices agree the whole code words agree, so the packed words must too
    same_rows = rows[~diff.any(1)]
    assert np.array_equal(g.codes[same_rows], e.codes[same_rows]), "packed code words differ"
    return {"chunks": int(ok.sum()), "near_ties": int((ok & (gap < NEAR_TIE)).sum()),
            "index_mismatch_in_near_ties": int(diff.sum()), "outliers": int(e.n_out[-1])}


def compare_decode(out_gpu: np.ndarray, out_or: np.ndarray, r_hat: np.ndarray, flag: np.ndarray):
    """Reconstruction within RECON_TOL of the chunk norm (r_hat: the decoded norm; fp16
    rounding of a component is at most 2^-11 of it); flagged chunks bit-exact."""
    nc = flag.shape[-1]
    a = chunked(out_gpu, nc)
    b = chunked(out_or, nc)
    fl = flag.astype(bool)
    assert np.array_equal(a[fl], b[fl]), "restored outliers differ"
    af = a.view(np.float16).astype(np.float64)
    bf = b.view(np.float16).astype(np.float64)
    err = np.abs(af - bf).max(-1)
    bound = RECON_TOL * r_hat + 1e-12
    bad = (~fl) & (err > bound)
    assert not bad.any(), (np.argwhere(bad)[:5], err[bad][:5], r_hat[bad][:5])
    return float((err[~fl] / np.maximum(r_hat[~fl], 1e-30)).max()) if (~fl).any() else 0.0
