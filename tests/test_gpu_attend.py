"""GPU parity of the attention entry points (single-query attention read from the packed K and V caches,
paper App. F) against the fp64 oracle: the oracle decodes K and V from the SAME encoded bytes to fp16
(its own decode), takes the plain softmax attention over them in fp64, and the library's fp16 output
must agree within a bound derived per output element (see _check): one fp16 rounding of the result;
the elements of K_hat and V_hat whose exact reconstruction lies so close to the midpoint between two
fp16 values that the library's fp32 arithmetic may round them the other way (found from the oracle's
unrounded decode, and weighted by the softmax weights they carry); and ATT_TOL = 1e-4 of the weighted
sum of |V_hat| for the fp32 arithmetic of the attention itself (score sums, exp2, 22-bit weights,
running sums over T terms).  The observed error is printed."""
from __future__ import annotations

import math

import numpy as np
import pytest
import torch

import oracle
import paper_2605_27646_amd as hq
import workloads
from gpu_util import gpu_encode, upload_encoded

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
ATT_TOL = 1e-4


@pytest.fixture(params=["form_by_size", "form_with_tables"], autouse=True)
def attend_form(request, monkeypatch):
    """Every test of this file runs twice: with the form of the attention that the library picks by the size
    of the cache, and with the form that reads the reconstruction from per-head tables in LDS asked for through
    HQMQ_FLAG_ATTEND_TABLES (taken whenever the tables fit).  Same bound for both."""
    if request.param == "form_with_tables":
        def flagged(fn):
            def call(params, *args, **kwargs):
                p = hq.HqmqParams.from_buffer_copy(params)
                p.flags |= hq.HQMQ_FLAG_ATTEND_TABLES
                return fn(p, *args, **kwargs)
            return call
        for name in ("hqmq_attend", "hqmq_attend_lse", "hqmq_attend_masked", "hqmq_attend_workspace_bytes"):
            monkeypatch.setattr(hq, name, flagged(getattr(hq, name)))
    return request.param


def _bits(x: torch.Tensor) -> np.ndarray:
    return x.contiguous().cpu().numpy().view(np.uint16)


def _secs(seed, H, S):
    cb = hq.hqmq_build_codebooks(seed, 1, H, S)
    return cb[0, 0].contiguous(), cb[0, 1].contiguous()


def _query(B, Hq, seed, gain=1.0, D=128):
    gen = torch.Generator().manual_seed(seed)
    return (torch.randn(B, Hq, D, generator=gen) * gain).to(torch.float16)


def _gpu_attend(params, q, scale, bufs_k, sec_k, bufs_v, sec_v):
    q_dev = q.to(DEV)
    out = torch.full_like(q_dev, float("nan"))
    ws = torch.empty(hq.hqmq_attend_workspace_bytes(params, q.shape[1]), dtype=torch.uint8, device=DEV)
    ws.fill_(0xCD)                      # the workspace needs no initialisation
    hq.hqmq_attend(params, q_dev, scale, bufs_k, sec_k, bufs_v, sec_v, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


class Decoded:
    """A cache tensor as the oracle decodes it: `hat` = the fp16 values widened to fp64 [B, H, T, D];
    `slack` = for every element the fp16 spacing if it could have rounded to the neighbouring value,
    else 0.  The library reconstructs in fp32 and the oracle in fp64 before the same fp16 rounding; the
    fp32 value is off by at most 6e-7 of the chunk's norm (six roundings of products bounded by it), so
    an element whose exact value lies that close to the midpoint between two fp16 values may land on
    either side (the decode's own tolerance allows exactly that), and no other element can."""

    def __init__(self, e, sec_np, B, H, T, b_r, D=128):
        args = (e.codes, e.sigma, e.flags, e.row_off, e.outliers, sec_np, B, H, T, b_r)
        bits, r_hat = oracle.decode(*args, True, D=D)
        exact = oracle.decode64(*args, D=D)
        h16 = bits.view(np.float16).reshape(B, H, T, D)
        self.hat = h16.astype(np.float64)
        ulp = np.spacing(np.abs(h16)).astype(np.float64)
        nc = r_hat.shape[-1]
        r_el = np.repeat(r_hat.reshape(B, H, T, nc), 4, axis=-1)[..., :D]
        to_mid = 0.5 * ulp - np.abs(exact - self.hat)
        self.slack = np.where(to_mid <= 6e-7 * r_el, ulp, 0.0)


def _decoded(e, sec_np, B, H, T, b_r, D=128):
    return Decoded(e, sec_np, B, H, T, b_r, D)


def _weights(q, K, scale, visible):
    """Softmax weights of the oracle's scores, plain numpy: [B, H, G, T]."""
    B, Hq, D = q.shape
    H, T = K.hat.shape[1], K.hat.shape[2]
    qf = q.numpy().astype(np.float64).reshape(B, H, Hq // H, D)
    s = np.einsum("bhgd,bhtd->bhgt", qf, K.hat) * scale
    if visible is not None:
        seen = np.arange(T)[None, None, None, :] < np.asarray(visible).reshape(B, H, Hq // H, 1)
        s = np.where(seen, s, -np.inf)
    m = s.max(-1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    p = np.exp(s - m)
    tot = p.sum(-1, keepdims=True)
    return p / np.where(tot > 0, tot, 1.0), qf


def _check(got, want64, K, V, q, scale, visible=None, lse=None, lse_want=None):
    """|got - want| against a bound derived per output element (first order in the small terms):
      2^-11 |o|                          the one fp16 rounding of the result
      sum_t p_t slack(v_td)              elements of V_hat that may have rounded the other way
      1.5 sum_t p_t delta_t (|v_td| + |o_d|)   elements of K_hat that may have: they move the score of row t
                                         by at most delta_t = scale sum_d |q_d| slack(k_td), and
                                         d o_d / d s_t = p_t (v_td - o_d)
      ATT_TOL sum_t p_t |v_td|           fp32 accumulation over T terms, 22-bit weights, exp2, score rounding
    and of the log-sum-exp, d lse / d s_t = p_t:  2e-5 max(1, |lse|) + 1.5 sum_t p_t delta_t."""
    B, Hq, D = q.shape
    H = K.hat.shape[1]
    p, qf = _weights(q, K, scale, visible)
    delta = scale * np.einsum("bhgd,bhtd->bhgt", np.abs(qf), K.slack)
    pd = p * delta
    absV = np.abs(V.hat)
    A = np.einsum("bhgt,bhtd->bhgd", p, absV).reshape(B, Hq, D)
    from_v = np.einsum("bhgt,bhtd->bhgd", p, V.slack).reshape(B, Hq, D)
    from_k = 1.5 * (np.einsum("bhgt,bhtd->bhgd", pd, absV).reshape(B, Hq, D)
                    + np.abs(want64) * pd.sum(-1).reshape(B, Hq, 1))
    bound = 2.0 ** -11 * np.abs(want64) * 1.001 + from_v + from_k + ATT_TOL * A + 2.0 ** -24
    err = np.abs(got - want64)
    assert np.isfinite(got).all()
    assert (err <= bound).all(), (float(err.max()), np.argwhere(err > bound)[:5], err[err > bound][:5], bound[err > bound][:5])
    rel = float((err / np.maximum(A, 1e-3 * A.max() + 1e-30)).max())   # reported only; tiny outputs sit on the fp16 floor
    print({"max_err_over_weighted_abs_v": rel, "k_may_flip": int((K.slack > 0).sum()), "v_may_flip": int((V.slack > 0).sum())},
          flush=True)
    if lse is not None:
        fin = np.isfinite(lse_want)
        assert np.array_equal(np.isneginf(lse), np.isneginf(lse_want))
        tol = 2e-5 * np.maximum(1.0, np.abs(np.where(fin, lse_want, 0.0))) + 1.5 * pd.sum(-1).reshape(B, Hq)
        diff = np.abs(lse[fin] - lse_want[fin])
        assert (diff <= tol[fin]).all(), float(diff.max())
    return rel


def _oracle_attend(enc, sec_np, q, scale, B, H, T, b_r, D=128):
    """enc: a pair of objects with codes / sigma / flags / row_off / outliers (numpy)."""
    K = _decoded(enc[0], sec_np[0], B, H, T, b_r, D)
    V = _decoded(enc[1], sec_np[1], B, H, T, b_r, D)
    _, o64 = oracle.attend(_bits(q), K.hat, V.hat, scale)
    return o64, K, V


def _tensors(B, H, T, seed, law_sigma=0.7, D=128):
    wl = workloads.Workload("att", 300 + seed, 1, B, H, T, D, 16, sigma_g=law_sigma)
    return workloads.make_tensor(wl, 0, 0, "cpu"), workloads.make_tensor(wl, 0, 1, "cpu")


@pytest.mark.parametrize("B,H,T,Hq,S,b_r", [
    (1, 1, 1, 1, 16, 6),          # a single cached token: the output is its value row
    (1, 2, 63, 4, 16, 6),         # ragged tile
    (2, 2, 200, 8, 64, 6),        # 4 query heads per kv head, several tiles
    (1, 1, 1000, 8, 24, 6),       # 8 query heads per kv head, S not a power of two
    (1, 1, 90, 16, 16, 6),        # 16 per kv head: every column of the product in use
    (1, 3, 129, 9, 256, 4),       # 3 per kv head, one row past a tile
    (1, 2, 777, 14, 48, 8),       # 7 per kv head (the Qwen-2.5-7B grouping)
    (1, 1, 150, 4, 700, 6),       # S past the matrix-core screen of the encode, not a power of two
    (1, 1, 100, 2, 2048, 6),      # the two tables of a head past 64 KiB of LDS
    (1, 1, 70, 16, 2730, 8),      # largest S with the largest merge buffer (16 query heads per kv head)
])
def test_attend_small_oracle_encoded(B, H, T, Hq, S, b_r):
    """Identical bytes on both sides: encoded by the oracle, uploaded."""
    k, v = _tensors(B, H, T, seed=T)
    sec_k, sec_v = _secs(5, H, S)
    ek = oracle.encode(_bits(k), sec_k.numpy(), b_r=b_r)
    ev = oracle.encode(_bits(v), sec_v.numpy(), b_r=b_r)
    assert ek.n_out[-1] > 0 or T < 8
    q = _query(B, Hq, seed=T + 1)
    scale = 1 / math.sqrt(128)
    want, Kd, Vd = _oracle_attend((ek, ev), (sec_k.numpy(), sec_v.numpy()), q, scale, B, H, T, b_r)
    params = hq.params_for(k.to(DEV), S, b_r)
    got = _gpu_attend(params, q, scale, upload_encoded(ek, DEV), sec_k.to(DEV), upload_encoded(ev, DEV),
                      sec_v.to(DEV))
    _check(got, want, Kd, Vd, q, scale)


@pytest.mark.parametrize("D,B,H,T,Hq,S,b_r", [
    (64, 1, 2, 63, 4, 16, 6),           # 16 chunks per row: 4 score products, one column group of values
    (64, 2, 1, 1000, 8, 192, 4),        # the paper's s192_r4, 8 query heads per kv head
    (64, 1, 1, 1, 16, 24, 4),           # a single cached token
    (96, 1, 2, 129, 6, 16, 6),          # 24 chunks per row: 6 score products, second column group half empty
    (96, 2, 2, 777, 8, 192, 4),
    (96, 1, 1, 3000, 16, 48, 3),
])
def test_attend_other_head_dimensions(D, B, H, T, Hq, S, b_r):
    """Heads of 64 and 96 elements, GPU-encoded (exercises their search and packing as well); the oracle
    reads those bytes back, decodes and attends."""
    k, v = _tensors(B, H, T, seed=T + D, D=D)
    sec_k, sec_v = _secs(7, H, S)
    gk = gpu_encode(k.to(DEV), sec_k.to(DEV), b_r)
    gv = gpu_encode(v.to(DEV), sec_v.to(DEV), b_r)
    assert gk.status == 0 and gv.status == 0 and (gk.n_out[-1] > 0 or T < 8)
    q = _query(B, Hq, seed=T + 2, gain=1.5, D=D)
    scale = 1 / math.sqrt(D)
    want, Kd, Vd = _oracle_attend((gk, gv), (sec_k.numpy(), sec_v.numpy()), q, scale, B, H, T, b_r, D)
    got = _gpu_attend(gk.params, q, scale, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    _check(got, want, Kd, Vd, q, scale)


def test_attend_other_head_dimensions_full_size_with_lse():
    """One layer of the 64-element workload at its full length, and the log-sum-exp output."""
    wl = workloads.WORKLOADS["gqa8_d64_32k"]
    k = workloads.make_tensor(wl, 0, 0, "cpu")
    v = workloads.make_tensor(wl, 0, 1, "cpu")
    sec_k, sec_v = _secs(0, wl.H, wl.S)
    gk = gpu_encode(k.to(DEV), sec_k.to(DEV), wl.b_r)
    gv = gpu_encode(v.to(DEV), sec_v.to(DEV), wl.b_r)
    Hq = 4 * wl.H
    q = _query(wl.B, Hq, seed=5, gain=2.0, D=wl.D)
    scale = 1 / math.sqrt(wl.D)
    Kd = _decoded(gk, sec_k.numpy(), wl.B, wl.H, wl.T, wl.b_r, wl.D)
    Vd = _decoded(gv, sec_v.numpy(), wl.B, wl.H, wl.T, wl.b_r, wl.D)
    _, want, lse_want = oracle.attend(_bits(q), Kd.hat, Vd.hat, scale, want_lse=True)
    q_dev = q.to(DEV)
    out = torch.full_like(q_dev, float("nan"))
    lse = torch.full((wl.B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(hq.hqmq_attend_workspace_bytes(gk.params, Hq), dtype=torch.uint8, device=DEV)
    hq.hqmq_attend_lse(gk.params, q_dev, scale, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV), out, lse, ws)
    torch.cuda.synchronize()
    _check(out.cpu().numpy().astype(np.float64), want, Kd, Vd, q, scale, lse=lse.cpu().numpy().astype(np.float64),
           lse_want=lse_want)


def test_attend_splits_with_several_tiles_each_gpu_encoded():
    """Long enough that every workgroup walks several tiles and the last split is ragged;
    encoded by the library, the oracle reads those bytes back."""
    B, H, T, Hq, S, b_r = 2, 4, 20011, 16, 16, 6
    k, v = _tensors(B, H, T, seed=9)
    sec_k, sec_v = _secs(6, H, S)
    gk = gpu_encode(k.to(DEV), sec_k.to(DEV), b_r)
    gv = gpu_encode(v.to(DEV), sec_v.to(DEV), b_r)
    assert gk.status == 0 and gv.status == 0 and gk.n_out[-1] > 0 and gv.n_out[-1] > 0
    q = _query(B, Hq, seed=10, gain=2.0)
    scale = 1 / math.sqrt(128)
    want, Kd, Vd = _oracle_attend((gk, gv), (sec_k.numpy(), sec_v.numpy()), q, scale, B, H, T, b_r)
    got = _gpu_attend(gk.params, q, scale, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    _check(got, want, Kd, Vd, q, scale)


def test_attend_picks_single_rows_including_outlier_rows():
    """A query aligned with one cached key and a large scale puts all the weight on that token:
    the output must be that token's reconstructed value row, outlier chunks included, to fp16
    rounding.  One query head per probed token, the probes spread over tiles and waves."""
    B, H, T, S, b_r = 1, 1, 517, 16, 6
    Hq = 8
    k, v = _tensors(B, H, T, seed=21, law_sigma=1.0)
    sec_k, sec_v = _secs(7, H, S)
    ek = oracle.encode(_bits(k), sec_k.numpy(), b_r=b_r)
    ev = oracle.encode(_bits(v), sec_v.numpy(), b_r=b_r)
    Kd = _decoded(ek, sec_k.numpy(), B, H, T, b_r)
    Vd = _decoded(ev, sec_v.numpy(), B, H, T, b_r)
    K64, V64 = Kd.hat, Vd.hat
    # a row with a large key norm wins a scaled dot product against its own direction: take the
    # largest of each eighth of the sequence, so the probes fall into different tiles and waves
    norms = np.linalg.norm(K64[0, 0], axis=1)
    edges = np.linspace(0, T, Hq + 1).astype(int)
    probes = [int(lo + np.argmax(norms[lo:hi])) for lo, hi in zip(edges[:-1], edges[1:])]
    assert ev.flag.reshape(T, -1)[probes].any(1).sum() >= 4     # their value rows hold outlier chunks
    q = np.stack([K64[0, 0, t] / norms[t] for t in probes])[None]            # [1, 8, 128]
    q_t = torch.from_numpy(q).to(torch.float16)
    scale = 64.0
    want = oracle.attend(_bits(q_t), K64, V64, scale)[1]
    params = hq.params_for(k.to(DEV), S, b_r)
    got = _gpu_attend(params, q_t, scale, upload_encoded(ek, DEV), sec_k.to(DEV), upload_encoded(ev, DEV),
                      sec_v.to(DEV))
    # the probe really isolates one token in the oracle ...
    sel = [int(np.abs(want[0, i] - V64[0, 0]).sum(1).argmin()) for i in range(Hq)]
    iso = [np.abs(want[0, i] - V64[0, 0, sel[i]]).max() < 1e-6 * np.abs(V64[0, 0, sel[i]]).max() for i in range(Hq)]
    assert sum(iso) >= 4, iso
    # ... and the library returns that row to fp16 rounding
    for i in range(Hq):
        if iso[i]:
            row = V64[0, 0, sel[i]]
            assert np.abs(got[0, i] - row).max() <= 2.0 ** -10 * np.abs(row).max() + 1e-7, (i, sel[i])
    _check(got, want, Kd, Vd, q_t, scale)


def test_attend_without_outlier_lists():
    B, H, T, Hq, S, b_r = 1, 2, 300, 4, 16, 6
    k, v = _tensors(B, H, T, seed=31)
    sec_k, sec_v = _secs(8, H, S)
    flags = hq.HQMQ_FLAG_NO_OUTLIERS
    gk = gpu_encode(k.to(DEV), sec_k.to(DEV), b_r, flags=flags)
    gv = gpu_encode(v.to(DEV), sec_v.to(DEV), b_r, flags=flags)
    assert gk.bufs.outlier_capacity == 0 and gk.n_out[-1] == 0
    q = _query(B, Hq, seed=32)
    want, Kd, Vd = _oracle_attend((gk, gv), (sec_k.numpy(), sec_v.numpy()), q, 0.1, B, H, T, b_r)
    got = _gpu_attend(gk.params, q, 0.1, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    _check(got, want, Kd, Vd, q, 0.1)


def _spiky(B, H, T, seed, rows, big=5.0, small=0.01):
    """Small Gaussian rows with a band of large rows: every chunk of the band is an outlier."""
    gen = torch.Generator().manual_seed(seed)
    x = torch.randn(B, H, T, 128, generator=gen) * small
    x[:, :, rows[0]:rows[1]] = torch.randn(B, H, rows[1] - rows[0], 128, generator=gen) * big
    return x.to(torch.float16)


def test_attend_windows_larger_than_the_lds_slots():
    """16-row groups whose outlier window exceeds the slots kept in LDS (here: whole rows flagged)."""
    B, H, T, Hq, S, b_r = 1, 2, 200, 4, 16, 6
    k, v = _spiky(B, H, T, 61, (40, 60)), _spiky(B, H, T, 62, (35, 57))
    sec_k, sec_v = _secs(10, H, S)
    ek = oracle.encode(_bits(k), sec_k.numpy(), b_r=b_r)
    ev = oracle.encode(_bits(v), sec_v.numpy(), b_r=b_r)
    per_row = ek.flag.reshape(B * H, T, -1).sum(-1)
    assert per_row[:, 40:60].min() == 32 and per_row[0, 32:48].sum() > 128
    q = _query(B, Hq, seed=63, gain=3.0)
    want, Kd, Vd = _oracle_attend((ek, ev), (sec_k.numpy(), sec_v.numpy()), q, 0.3, B, H, T, b_r)
    params = hq.params_for(k.to(DEV), S, b_r)
    got = _gpu_attend(params, q, 0.3, upload_encoded(ek, DEV), sec_k.to(DEV), upload_encoded(ev, DEV),
                      sec_v.to(DEV))
    _check(got, want, Kd, Vd, q, 0.3)


def test_attend_with_truncated_outlier_lists():
    """An encode that overflowed its lists: the dropped outliers count as zeros, as in the decode."""
    B, H, T, Hq, S, b_r = 1, 2, 300, 4, 16, 6
    k, v = _tensors(B, H, T, seed=71, law_sigma=1.0)
    sec_k, sec_v = _secs(11, H, S)
    full_k = gpu_encode(k.to(DEV), sec_k.to(DEV), b_r)
    full_v = gpu_encode(v.to(DEV), sec_v.to(DEV), b_r)
    nk, nv = int(full_k.n_out[-1]), int(full_v.n_out[-1])
    gk = gpu_encode(k.to(DEV), sec_k.to(DEV), b_r, outlier_capacity=nk // 2)
    gv = gpu_encode(v.to(DEV), sec_v.to(DEV), b_r, outlier_capacity=nv // 3)
    assert gk.status & hq.HQMQ_STATUS_OUTLIER_OVERFLOW and gv.status & hq.HQMQ_STATUS_OUTLIER_OVERFLOW

    class Padded:                                   # the kept prefix, zeros for what was dropped
        def __init__(self, g, total):
            self.codes, self.sigma, self.flags, self.row_off = g.codes, g.sigma, g.flags, g.row_off
            self.outliers = np.zeros((total, 4), np.uint16)
            self.outliers[: g.outliers.shape[0]] = g.outliers
    q = _query(B, Hq, seed=72)
    want, Kd, Vd = _oracle_attend((Padded(gk, nk), Padded(gv, nv)), (sec_k.numpy(), sec_v.numpy()), q, 0.09,
                                  B, H, T, b_r)
    got = _gpu_attend(gk.params, q, 0.09, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    _check(got, want, Kd, Vd, q, 0.09)


def test_attend_scales_near_the_fp16_maximum():
    """Rows whose scale is close to 65504: the tile takes the saturating conversion."""
    B, H, T, Hq, S, b_r = 1, 1, 100, 2, 16, 6
    gen = torch.Generator().manual_seed(81)
    k = (torch.randn(B, H, T, 128, generator=gen) * 12000).clamp(-65504, 65504).to(torch.float16)
    v = (torch.randn(B, H, T, 128, generator=gen) * 12000).clamp(-65504, 65504).to(torch.float16)
    sec_k, sec_v = _secs(12, H, S)
    flags = hq.HQMQ_FLAG_NO_OUTLIERS
    gk = gpu_encode(k.to(DEV), sec_k.to(DEV), b_r, flags=flags)
    gv = gpu_encode(v.to(DEV), sec_v.to(DEV), b_r, flags=flags)
    assert (gk.sigma.view(np.float16).astype(np.float64) >= 32752).any()
    q = _query(B, Hq, seed=82)
    want, Kd, Vd = _oracle_attend((gk, gv), (sec_k.numpy(), sec_v.numpy()), q, 1e-5, B, H, T, b_r)
    got = _gpu_attend(gk.params, q, 1e-5, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    _check(got, want, Kd, Vd, q, 1e-5)


def test_attend_llama3_8b_32k_layer_full_size():
    """The bench's shape (T = 32768, 8 kv heads, 32 query heads): encoded by the library, every
    output element checked against the oracle's attention over the same bytes."""
    wl = workloads.WORKLOADS["llama3_8b_32k"]
    k = workloads.make_tensor(wl, 3, 0, DEV)
    v = workloads.make_tensor(wl, 3, 1, DEV)
    cb = hq.hqmq_build_codebooks(0, 4, wl.H, wl.S)
    sec_k, sec_v = cb[3, 0].contiguous(), cb[3, 1].contiguous()
    gk = gpu_encode(k, sec_k.to(DEV), wl.b_r)
    gv = gpu_encode(v, sec_v.to(DEV), wl.b_r)
    Hq = 32
    q = _query(wl.B, Hq, seed=40, gain=1.5)
    scale = 1 / math.sqrt(128)
    want, Kd, Vd = _oracle_attend((gk, gv), (sec_k.numpy(), sec_v.numpy()), q, scale, wl.B, wl.H, wl.T, wl.b_r)
    got = _gpu_attend(gk.params, q, scale, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    _check(got, want, Kd, Vd, q, scale)


def test_attend_128k_tokens_one_query_head_per_kv_head():
    """The longest workload shape (T = 131072, 8 kv heads), G = 1: 32 tiles per split."""
    wl = workloads.WORKLOADS["llama3_70b_128k"]
    k = workloads.make_tensor(wl, 1, 0, DEV)
    v = workloads.make_tensor(wl, 1, 1, DEV)
    cb = hq.hqmq_build_codebooks(0, 2, wl.H, wl.S)
    sec_k, sec_v = cb[1, 0].contiguous(), cb[1, 1].contiguous()
    gk = gpu_encode(k, sec_k.to(DEV), wl.b_r)
    gv = gpu_encode(v, sec_v.to(DEV), wl.b_r)
    del k, v
    q = _query(wl.B, wl.H, seed=90, gain=2.0)
    scale = 1 / math.sqrt(128)
    want, Kd, Vd = _oracle_attend((gk, gv), (sec_k.numpy(), sec_v.numpy()), q, scale, wl.B, wl.H, wl.T, wl.b_r)
    got = _gpu_attend(gk.params, q, scale, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    _check(got, want, Kd, Vd, q, scale)


def test_attend_is_deterministic():
    B, H, T, Hq, S = 1, 2, 5000, 8, 16
    k, v = _tensors(B, H, T, seed=51)
    sec_k, sec_v = _secs(9, H, S)
    gk = gpu_encode(k.to(DEV), sec_k.to(DEV))
    gv = gpu_encode(v.to(DEV), sec_v.to(DEV))
    q = _query(B, Hq, seed=52)
    a = _gpu_attend(gk.params, q, 0.09, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    b = _gpu_attend(gk.params, q, 0.09, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    assert np.array_equal(a, b)


def test_attend_lse_combines_a_prefill_tensor_and_appended_tokens():
    """The generation setting end to end: a prefill tensor encoded with its own medians, then two batches
    of appended tokens encoded against the prefill's thresholds as tensors of their own.  One attention
    call per tensor with its log-sum-exp; the lse-weighted combination must equal the oracle's attention
    over the concatenation of the three decoded ranges, and each lse the oracle's."""
    B, H, Hq, S, b_r = 2, 2, 8, 16, 6
    T_parts = (700, 5, 64)
    k_all, v_all = _tensors(B, H, sum(T_parts), seed=77)
    sec_k, sec_v = _secs(8, H, S)
    sec_np = (sec_k.numpy(), sec_v.numpy())
    sec_dev = (sec_k.to(DEV), sec_v.to(DEV))
    q = _query(B, Hq, seed=78, gain=1.5)
    scale = 1 / math.sqrt(128)
    bounds = np.cumsum((0,) + T_parts)
    outs, lses, K64s, V64s = [], [], [], []
    thr = [None, None]
    for i, (a, b) in enumerate(zip(bounds[:-1], bounds[1:])):
        encs = []
        for role, x_all in enumerate((k_all, v_all)):
            x = x_all[:, :, a:b].contiguous().to(DEV)
            p = hq.params_for(x, S, b_r)
            ws = hq.alloc_workspace(p, DEV)
            if i == 0:
                bufs = hq.alloc_encoded(p, DEV)
                hq.hqmq_encode(p, x, sec_dev[role], bufs, ws)
                thr[role] = hq.hqmq_thresholds(p, ws)
            else:
                bufs = hq.alloc_encoded(p, DEV, outlier_capacity=B * H * (b - a) * 32)
                hq.hqmq_encode_given_thresholds(p, x, sec_dev[role], thr[role], bufs, ws)
            torch.cuda.synchronize()
            assert int(bufs.status.item()) == 0
            encs.append((p, bufs))
        p = encs[0][0]
        q_dev = q.to(DEV)
        out = torch.full_like(q_dev, float("nan"))
        lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
        ws = torch.empty(hq.hqmq_attend_workspace_bytes(p, Hq), dtype=torch.uint8, device=DEV)
        hq.hqmq_attend_lse(p, q_dev, scale, encs[0][1], sec_dev[0], encs[1][1], sec_dev[1], out, lse, ws)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy().astype(np.float64))
        lses.append(lse.cpu().numpy().astype(np.float64))
        # the oracle reads the library's bytes of this range back
        def host(bufs):
            total = int(bufs.n_outliers[-1].item())
            class E:
                pass
            e = E()
            e.codes = bufs.codes.cpu().numpy().view(np.uint32); e.sigma = bufs.sigma.cpu().numpy().view(np.uint16)
            e.flags = bufs.flags.cpu().numpy().view(np.uint32); e.row_off = bufs.row_off.cpu().numpy().view(np.uint32)
            e.outliers = bufs.outliers[:total].cpu().numpy().view(np.uint16).reshape(total, 4)
            return e
        K64s.append(_decoded(host(encs[0][1]), sec_np[0], B, H, b - a, b_r))
        V64s.append(_decoded(host(encs[1][1]), sec_np[1], B, H, b - a, b_r))
        _, want_i, lse_i = oracle.attend(_bits(q), K64s[-1].hat, V64s[-1].hat, scale, want_lse=True)
        _check(outs[-1], want_i, K64s[-1], V64s[-1], q, scale, lse=lses[-1], lse_want=lse_i)
    Kd, Vd = K64s[0], V64s[0]       # the whole cache: the three ranges side by side
    Kd.hat = np.concatenate([k_.hat for k_ in K64s], axis=2)
    Kd.slack = np.concatenate([k_.slack for k_ in K64s], axis=2)
    Vd.hat = np.concatenate([v_.hat for v_ in V64s], axis=2)
    Vd.slack = np.concatenate([v_.slack for v_ in V64s], axis=2)
    _, want, lse_want = oracle.attend(_bits(q), Kd.hat, Vd.hat, scale, want_lse=True)
    L = np.logaddexp.reduce(np.stack(lses), axis=0)
    merged = sum(np.exp(l - L)[..., None] * o for l, o in zip(lses, outs))
    # the combination of the parts against the whole: every part carries its own fp16 rounding (their
    # weights sum to one), the rest of the bound is the whole cache's
    p, _ = _weights(q, Kd, scale, None)
    A = np.einsum("bhgt,bhtd->bhgd", p, np.abs(Vd.hat)).reshape(B, Hq, 128)
    pd_sum = 1.5 * (p * scale * np.einsum("bhgd,bhtd->bhgt", np.abs(q.numpy().astype(np.float64)).reshape(B, H, Hq // H, 128),
                                          Kd.slack)).sum(-1).reshape(B, Hq)
    assert (np.abs(L - lse_want) <= 2e-5 * np.maximum(1.0, np.abs(lse_want)) + pd_sum).all()
    # each part's output was rounded to fp16 on its own: |part| <= A / weight, so 2^-11 A in total per part
    err = np.abs(merged - want)
    slack_v = np.einsum("bhgt,bhtd->bhgd", p, Vd.slack).reshape(B, Hq, 128)
    assert (err <= len(outs) * 2.0 ** -11 * A + slack_v + (ATT_TOL + 3 * pd_sum[..., None]) * A + 2.0 ** -24).all(), float(err.max())


@pytest.mark.parametrize("D,T,n_tok,G", [(128, 3001, 4, 4), (64, 700, 16, 1), (96, 130, 2, 7)])
def test_attend_causal_limit_for_several_query_tokens(D, T, n_tok, G):
    """A step with n_tok query tokens per sequence riding as extra query heads of their kv head: token i
    sees the cache up to its own position, T - n_tok + i + 1 tokens."""
    B, H, S, b_r = 2, 2, 24, 4
    k, v = _tensors(B, H, T, seed=T + n_tok, D=D)
    sec_k, sec_v = _secs(9, H, S)
    gk = gpu_encode(k.to(DEV), sec_k.to(DEV), b_r)
    gv = gpu_encode(v.to(DEV), sec_v.to(DEV), b_r)
    Hq = H * n_tok * G                                   # laid out [H][token][head of the group]
    q = _query(B, Hq, seed=3 * T, gain=1.5, D=D)
    vis = np.zeros((B, H, n_tok, G), np.int32)
    vis[:] = (T - n_tok + 1 + np.arange(n_tok))[None, None, :, None]
    vis = vis.reshape(B, Hq)
    scale = 1 / math.sqrt(D)
    Kd = _decoded(gk, sec_k.numpy(), B, H, T, b_r, D)
    Vd = _decoded(gv, sec_v.numpy(), B, H, T, b_r, D)
    _, want, lse_want = oracle.attend(_bits(q), Kd.hat, Vd.hat, scale, want_lse=True, visible=vis)
    q_dev = q.to(DEV)
    out = torch.full_like(q_dev, float("nan"))
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(hq.hqmq_attend_workspace_bytes(gk.params, Hq), dtype=torch.uint8, device=DEV)
    hq.hqmq_attend_masked(gk.params, q_dev, scale, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV),
                          torch.from_numpy(vis).to(DEV), out, ws, lse)
    torch.cuda.synchronize()
    _check(out.cpu().numpy().astype(np.float64), want, Kd, Vd, q, scale, visible=vis,
           lse=lse.cpu().numpy().astype(np.float64), lse_want=lse_want)


def test_attend_causal_limit_edge_values():
    """Limits of 0 (sees nothing: zeros, lse = -inf), 1, exactly T, beyond T, and limits that end inside a
    tile or exactly on a split boundary."""
    B, H, T, S, b_r, Hq = 1, 1, 20011, 16, 6, 16
    k, v = _tensors(B, H, T, seed=31)
    sec_k, sec_v = _secs(2, H, S)
    gk = gpu_encode(k.to(DEV), sec_k.to(DEV), b_r)
    gv = gpu_encode(v.to(DEV), sec_v.to(DEV), b_r)
    q = _query(B, Hq, seed=32, gain=2.0)
    vis = np.array([[0, 1, 2, 15, 16, 17, 63, 64, 65, 1024, 9999, 10048, T - 1, T, T + 5, 2 ** 31 - 1]], np.int32)
    scale = 1 / math.sqrt(128)
    Kd = _decoded(gk, sec_k.numpy(), B, H, T, b_r)
    Vd = _decoded(gv, sec_v.numpy(), B, H, T, b_r)
    _, want, lse_want = oracle.attend(_bits(q), Kd.hat, Vd.hat, scale, want_lse=True, visible=vis)
    q_dev = q.to(DEV)
    out = torch.full_like(q_dev, float("nan"))
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(hq.hqmq_attend_workspace_bytes(gk.params, Hq), dtype=torch.uint8, device=DEV)
    hq.hqmq_attend_masked(gk.params, q_dev, scale, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV),
                          torch.from_numpy(vis).to(DEV), out, ws, lse)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    _check(got, want, Kd, Vd, q, scale, visible=vis, lse=lse.cpu().numpy().astype(np.float64), lse_want=lse_want)
    assert not got[0, 0].any() and lse[0, 0].item() == -math.inf


def _attend_sweep_cases(n, seed):
    """Seeded random attention cases: head dimension, codebook size, radius width, group size, lengths on and off
    the tile and split edges, query gain, and the three entry points (plain, log-sum-exp, causal limits)."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        D = int(rng.choice([128, 96, 64]))
        S = int(rng.choice([1, 3, 16, 24, 64, 100, 192, 256, 512]))
        b_r = int(rng.integers(1, 9))
        B, H, G = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 17))
        T = int(rng.choice([1, 2, 15, 16, 17, 63, 64, 65, 129, int(rng.integers(1, 6000)), int(rng.integers(1, 40000))]))
        if B * H * T * (D // 4) * 24 * S > 2e8:    # the GPU encodes; the oracle decodes and attends
            T = max(1, int(2e8 / (B * H * (D // 4) * 24 * S)))
        cases.append((D, S, b_r, B, H, G, T, float(rng.choice([0.5, 1.5, 3.0])), int(rng.integers(0, 3)),
                      float(rng.choice([0.4, 0.9])), int(rng.integers(1, 10 ** 6))))
    return cases


@pytest.mark.parametrize("D,S,b_r,B,H,G,T,gain,mode,law,seed", _attend_sweep_cases(24, seed=20261128))
def test_attend_randomized_sweep(D, S, b_r, B, H, G, T, gain, mode, law, seed):
    print(f"case D={D} S={S} b_r={b_r} B={B} H={H} G={G} T={T} gain={gain} mode={mode} law={law} seed={seed}", flush=True)
    rng = np.random.default_rng(seed)
    k, v = _tensors(B, H, T, seed=seed, D=D, law_sigma=law)
    sec_k, sec_v = _secs(seed % 50, H, S)
    gk, gv = gpu_encode(k.to(DEV), sec_k.to(DEV), b_r), gpu_encode(v.to(DEV), sec_v.to(DEV), b_r)
    Hq = H * G
    q = _query(B, Hq, seed=seed + 1, gain=gain, D=D)
    scale = 1 / math.sqrt(D)
    Kd, Vd = _decoded(gk, sec_k.numpy(), B, H, T, b_r, D), _decoded(gv, sec_v.numpy(), B, H, T, b_r, D)
    vis = rng.integers(0, T + 3, (B, Hq)).astype(np.int32) if mode == 2 else None
    _, want, lse_want = oracle.attend(_bits(q), Kd.hat, Vd.hat, scale, want_lse=True, visible=vis)
    q_dev = q.to(DEV)
    out = torch.full_like(q_dev, float("nan"))
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(hq.hqmq_attend_workspace_bytes(gk.params, Hq), dtype=torch.uint8, device=DEV)
    ws.fill_(0xCD)
    args = (gk.params, q_dev, scale, gk.bufs, sec_k.to(DEV), gv.bufs, sec_v.to(DEV))
    if mode == 0:
        hq.hqmq_attend(*args, out, ws)
    elif mode == 1:
        hq.hqmq_attend_lse(*args, out, lse, ws)
    else:
        hq.hqmq_attend_masked(*args, torch.from_numpy(vis).to(DEV), out, ws, lse)
    torch.cuda.synchronize()
    _check(out.cpu().numpy().astype(np.float64), want, Kd, Vd, q, scale, visible=vis,
           lse=lse.cpu().numpy().astype(np.float64) if mode else None, lse_want=lse_want if mode else None)
