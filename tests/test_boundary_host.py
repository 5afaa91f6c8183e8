"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports every
symbol the header declares, validates its arguments, sizes its buffers, and builds the same
codebooks as the oracle's independent generator."""
import ctypes as C
import os
import re

import numpy as np
import pytest
import torch

import oracle
import paper_2605_27646_amd as hq
from paper_2605_27646_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hq.library_path()):
        from paper_2605_27646_amd import build
        build.build()
    return binding._load()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "hqmq.h")).read()
    declared = set(re.findall(r"^(?:int32_t|void|uint64_t)\s+(hqmq_\w+)\s*\(", header, re.M))
    assert declared == {"hqmq_build_codebooks", "hqmq_sizes", "hqmq_encode", "hqmq_encode_timed", "hqmq_encode_batch", "hqmq_encode_given_thresholds", "hqmq_encode_batch_given_thresholds", "hqmq_thresholds", "hqmq_shard_median_pass", "hqmq_shard_median_region", "hqmq_decode", "hqmq_decode_batch", "hqmq_attend", "hqmq_attend_lse", "hqmq_attend_masked", "hqmq_attend_workspace_bytes", "hqmq_last_hip_error", "hqmq_init", "hqmq_encode_static"}
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layouts_match_header():
    assert C.sizeof(hq.HqmqParams) == 56
    assert C.sizeof(hq.HqmqSizeInfo) == 96
    assert C.sizeof(binding._Encoded) == 56


def _params(**kw):
    d = dict(B=1, H=8, T=1024, D=128, stride_b=8 * 1024 * 128, stride_h=1024 * 128, stride_t=128, S=256,
             b_r=6, C=3.0, flags=0)
    d.update(kw)
    return hq.HqmqParams(**d)


def test_sizes_of_the_headline_workload(lib):
    info = hq.hqmq_sizes(_params(T=32768, stride_b=8 * 32768 * 128, stride_h=32768 * 128))
    assert info.n_rows == 8 * 32768
    assert (info.index_bits, info.code_bits) == (13, 19)           # ceil(log2(24*256)) + 6
    assert info.code_bytes == info.n_rows * 19 * 4
    assert info.sigma_bytes == info.n_rows * 2 and info.flag_bytes == info.n_rows * 4
    assert info.row_off_bytes == (info.n_rows + 1) * 4 and info.n_outliers_bytes == 36
    assert info.outlier_capacity_max == 8 * (32768 * 32 // 2)      # at most half of a head lies above its median
    assert info.outlier_bytes_max == info.outlier_capacity_max * 8
    assert 0 < info.workspace_bytes < 4 << 20
    # stored bits per element agree with the accounting of Sec. 3 taken with ceil(log2(24 S))
    stored = (info.code_bytes + info.sigma_bytes) * 8 / (info.n_rows * 128)
    assert stored == oracle.bits_per_element(256, 6, 128, stored=True)
    assert hq.hqmq_sizes(_params(C=0.5)).outlier_capacity_max == 8 * 1024 * 32
    assert hq.hqmq_sizes(_params(flags=hq.HQMQ_FLAG_NO_OUTLIERS)).outlier_capacity_max == 0


@pytest.mark.parametrize("D,S,b_r", [(64, 192, 4), (96, 192, 4), (96, 24, 3), (45, 48, 4), (4, 16, 6), (1, 1, 1),
                                     (128, 192, 6)])
def test_sizes_of_other_head_dimensions(lib, D, S, b_r):
    """Rows of ceil(D / 4) chunks packed into ceil(chunks * w / 32) words; any strides are accepted."""
    B, H, T = 2, 4, 100
    pitch = D + 3 if D != 128 else 128
    info = hq.hqmq_sizes(_params(B=B, H=H, T=T, D=D, S=S, b_r=b_r, stride_t=pitch, stride_h=T * pitch,
                                 stride_b=H * T * pitch))
    nc = -(-D // 4)
    w = oracle.index_bits(S) + b_r
    assert (info.chunks_per_row, info.code_bits, info.code_words_per_row) == (nc, w, -(-nc * w // 32))
    assert info.code_words_per_row == oracle.row_words(D, w)
    assert info.code_bytes == B * H * T * info.code_words_per_row * 4
    assert info.outlier_capacity_max == H * (B * T * nc // 2)
    # stored code + scale bits per element: the accounting of Sec. 3 with the index width rounded up
    # to whole bits, the padding of App. "Padding wrapper" and the row rounded up to whole words
    stored = (info.code_bytes + info.sigma_bytes) * 8 / (info.n_rows * D)
    ideal = oracle.bits_per_element(S, b_r, D, stored=True)
    padded = (ideal - 16 / D) * (1 + oracle.padding_overhead(D)) + 16 / D
    assert padded <= stored < padded + 32 / D


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), -1), (dict(T=-3), -1), (dict(stride_t=132), -1), (dict(stride_t=64), -1), (dict(stride_h=-8), -1),
    (dict(D=132, stride_t=136), -2), (dict(D=130), -2), (dict(D=0), -1), (dict(D=96, stride_t=64), -1), (dict(S=0), -2), (dict(S=2731), -2), (dict(b_r=0), -2), (dict(b_r=9), -2),
    (dict(C=0.0), -2), (dict(C=float("nan")), -2), (dict(C=float("inf")), -2), (dict(B=70000, H=1), -2),
    (dict(T=1 << 27), -2),
])
def test_sizes_rejects_bad_params(lib, kw, code):
    with pytest.raises(hq.HqmqError) as ei:
        hq.hqmq_sizes(_params(**kw))
    assert ei.value.code == code
    info = hq.HqmqSizeInfo()
    assert lib.hqmq_sizes(None, C.byref(info)) == -1
    assert lib.hqmq_sizes(C.byref(_params()), None) == -1


def test_encode_decode_reject_bad_arguments_without_touching_the_gpu(lib):
    p = _params()
    info = hq.hqmq_sizes(p)
    good = binding._Encoded(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    ws = int(info.workspace_bytes)
    enc = lib.hqmq_encode
    assert enc(None, 0x1000, 0x1000, C.byref(good), 0, 0x1000, ws, None) == -1
    assert enc(C.byref(p), None, 0x1000, C.byref(good), 0, 0x1000, ws, None) == -1          # null x
    assert enc(C.byref(p), 0x1008, 0x1000, C.byref(good), 0, 0x1000, ws, None) == -1        # misaligned x
    assert enc(C.byref(p), 0x1000, 0x1004, C.byref(good), 0, 0x1000, ws, None) == -1        # misaligned codebook
    assert enc(C.byref(p), 0x1000, 0x1000, None, 0, 0x1000, ws, None) == -1                 # null struct
    assert enc(C.byref(p), 0x1000, 0x1000, C.byref(good), 0, 0x1010, ws, None) == -1        # misaligned workspace
    assert enc(C.byref(p), 0x1000, 0x1000, C.byref(good), 0, 0x1000, ws - 1, None) == -3    # workspace too small
    bad = binding._Encoded(0x1000, 0x1000, None, 0x1000, 0x1000, 0x1000, 0x1000)
    assert enc(C.byref(p), 0x1000, 0x1000, C.byref(bad), 0, 0x1000, ws, None) == -1         # null member
    bad = binding._Encoded(0x1002, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    assert enc(C.byref(p), 0x1000, 0x1000, C.byref(bad), 0, 0x1000, ws, None) == -1         # misaligned member
    assert enc(C.byref(_params(D=132, stride_t=136)), 0x1000, 0x1000, C.byref(good), 0, 0x1000, ws, None) == -2
    es = lib.hqmq_encode_static
    assert es(C.byref(p), None, 0x1000, C.byref(good), 0, None) == -1                          # null x
    assert es(C.byref(p), 0x1000, 0x1000, C.byref(bad), 0, None) == -1                         # misaligned member
    wide = _params(H=64, stride_b=64 * 1024 * 128)                                             # 64 heads: 21 MiB of workspace
    assert hq.hqmq_sizes(wide).workspace_bytes > hq.HQMQ_STATIC_SCRATCH_BYTES
    assert es(C.byref(wide), 0x1000, 0x1000, C.byref(good), 0, None) == -3                     # beyond the static array
    assert hq.hqmq_sizes(_params(H=48, stride_b=48 * 1024 * 128)).workspace_bytes <= hq.HQMQ_STATIC_SCRATCH_BYTES
    dec = lib.hqmq_decode
    assert dec(C.byref(p), C.byref(good), 0, None, 0x1000, None) == -1
    assert dec(C.byref(p), C.byref(good), 0, 0x1000, 0x1008, None) == -1
    assert dec(C.byref(p), None, 0, 0x1000, 0x1000, None) == -1
    assert dec(C.byref(_params(S=2731)), C.byref(good), 0, 0x1000, 0x1000, None) == -2
    db = lib.hqmq_decode_batch
    encs = (binding._Encoded * 2)(good, good)
    caps = (C.c_uint64 * 2)(0, 0)
    ptrs = (C.c_void_p * 2)(0x1000, 0x1000)
    bad_ptrs = (C.c_void_p * 2)(0x1000, 0x1008)
    assert db(C.byref(p), 0, encs, caps, ptrs, ptrs, None) == -1                              # empty batch
    assert db(C.byref(p), 2, None, caps, ptrs, ptrs, None) == -1
    assert db(C.byref(p), 2, encs, None, ptrs, ptrs, None) == -1
    assert db(C.byref(p), 2, encs, caps, ptrs, bad_ptrs, None) == -1                          # second out misaligned
    assert db(C.byref(_params(b_r=0)), 2, encs, caps, ptrs, ptrs, None) == -2
    eb = lib.hqmq_encode_batch
    ws2 = 2 * ws
    assert eb(C.byref(p), 0, ptrs, ptrs, encs, caps, 0x1000, ws2, None, None) == -1                # empty batch
    assert eb(C.byref(p), 2, None, ptrs, encs, caps, 0x1000, ws2, None, None) == -1
    assert eb(C.byref(p), 2, ptrs, bad_ptrs, encs, caps, 0x1000, ws2, None, None) == -1            # second sec misaligned
    assert eb(C.byref(p), 2, ptrs, ptrs, encs, caps, 0x1000, ws2 - 1, None, None) == -3            # one slice per tensor
    assert eb(C.byref(p), 2, ptrs, ptrs, encs, caps, 0x1010, ws2, None, None) == -1                # workspace alignment
    eg = lib.hqmq_encode_given_thresholds
    assert eg(C.byref(p), 0x1000, 0x1000, None, C.byref(good), 0, 0x1000, ws, None) == -1          # no thresholds
    assert eg(C.byref(p), 0x1000, 0x1000, 0x1004, C.byref(good), 0, 0x1000, ws, None) == -1        # misaligned
    assert eg(C.byref(_params(flags=hq.HQMQ_FLAG_NO_OUTLIERS)), 0x1000, 0x1000, 0x1000, C.byref(good), 0, 0x1000,
              ws, None) == -1
    assert eg(C.byref(p), None, 0x1000, 0x1000, C.byref(good), 0, 0x1000, ws, None) == -1
    ebg = lib.hqmq_encode_batch_given_thresholds
    assert ebg(C.byref(p), 2, ptrs, ptrs, None, encs, caps, 0x1000, ws2, None) == -1
    assert ebg(C.byref(p), 2, ptrs, ptrs, (C.c_void_p * 2)(0x1000, None), encs, caps, 0x1000, ws2, None) == -1
    assert ebg(C.byref(p), 2, ptrs, ptrs, ptrs, encs, caps, 0x1000, ws2 - 1, None) == -3
    th = lib.hqmq_thresholds
    assert th(C.byref(p), None, ws, 0, 0x1000, None) == -1 and th(C.byref(p), 0x1000, ws, 0, None, None) == -1
    assert th(C.byref(p), 0x1000, 32 * ws, 32, 0x1000, None) == -1 and th(C.byref(p), 0x1000, ws, -1, 0x1000, None) == -1
    assert th(C.byref(_params(D=132, stride_t=136)), 0x1000, ws, 0, 0x1000, None) == -2
    assert th(C.byref(p), 0x1000, ws - 1, 0, 0x1000, None) == -3     # slice 0 does not fit the workspace
    assert th(C.byref(p), 0x1000, 3 * ws, 3, 0x1000, None) == -3     # slice 3 needs four slices
    sm = lib.hqmq_shard_median_pass
    own = 1024 * 32
    assert sm(C.byref(p), own, 0, None, 0x1000, ws, None) == -1 and sm(C.byref(p), own, 0, 0x1000, None, ws, None) == -1
    assert sm(C.byref(p), own, 7, 0x1000, 0x1000, ws, None) == -1 and sm(C.byref(p), own, -1, 0x1000, 0x1000, ws, None) == -1
    assert sm(C.byref(p), own - 1, 0, 0x1000, 0x1000, ws, None) == -1       # fewer chunks in total than this shard holds
    assert sm(C.byref(p), 1 << 32, 0, 0x1000, 0x1000, ws, None) == -2       # ranks are 32-bit
    assert sm(C.byref(p), own, 0, 0x1000, 0x1000, ws - 1, None) == -3
    assert sm(C.byref(_params(flags=hq.HQMQ_FLAG_NO_OUTLIERS)), own, 0, 0x1000, 0x1000, ws, None) == -1
    off, cnt = C.c_uint64(), C.c_uint64()
    reg = lib.hqmq_shard_median_region
    assert reg(C.byref(p), 0, C.byref(off), C.byref(cnt)) == 0 and cnt.value == 8 * 8192 and off.value % 256 == 0
    first = off.value
    assert reg(C.byref(p), 3, C.byref(off), C.byref(cnt)) == 0 and cnt.value == 8 * 1024 and off.value != first
    assert off.value + 4 * cnt.value <= ws
    assert reg(C.byref(p), 6, C.byref(off), C.byref(cnt)) == -1 and reg(C.byref(p), 0, None, C.byref(cnt)) == -1
    att = lib.hqmq_attend
    wsb = lib.hqmq_attend_workspace_bytes
    need = wsb(C.byref(p), 4 * p.H)
    assert need > 0 and need % 256 == 0
    assert wsb(C.byref(p), p.H + 1) == 0 and wsb(C.byref(p), 17 * p.H) == 0 and wsb(None, 4) == 0
    def call(params=p, hq_=4 * p.H, q=0x1000, scale=0.1, ek=good, ev=good, sk=0x1000, sv=0x1000, out=0x2000,
             ws_ptr=0x4000, ws_bytes=need):
        return att(C.byref(params), hq_, q, scale, C.byref(ek), 0, sk, C.byref(ev), 0, sv, out, ws_ptr,
                   ws_bytes, None)
    assert call(hq_=p.H + 1) == -1                    # not a multiple of the kv heads
    assert call(hq_=17 * p.H) == -2                   # more than 16 query heads per kv head
    assert call(q=None) == -1 and call(out=0x2008) == -1 and call(sv=None) == -1
    assert call(scale=float("nan")) == -1
    assert call(ek=bad) == -1 and call(ev=bad) == -1
    assert call(ws_ptr=0x4010) == -1                  # workspace not 256-byte aligned
    assert call(ws_bytes=need - 1) == -3
    assert call(params=_params(D=32)) == -2          # the attention kernel takes heads of 64, 96 or 128 elements
    am = lib.hqmq_attend_masked
    assert am(C.byref(p), 4 * p.H, 0x1000, 0.1, C.byref(good), 0, 0x1000, C.byref(good), 0, 0x1000, None, 0x2000, None,
              0x4000, need, None) == -1           # no visible array
    assert am(C.byref(p), 4 * p.H, 0x1000, 0.1, C.byref(good), 0, 0x1000, C.byref(good), 0, 0x1000, 0x3002, 0x2000, None,
              0x4000, need, None) == -1           # misaligned visible array
    assert am(C.byref(p), 4 * p.H, 0x1000, 0.1, C.byref(good), 0, 0x1000, C.byref(good), 0, 0x1000, 0x3000, 0x2000, None,
              0x4000, need - 1, None) == -3
    al = lib.hqmq_attend_lse
    assert al(C.byref(p), 4 * p.H, 0x1000, 0.1, C.byref(good), 0, 0x1000, C.byref(good), 0, 0x1000, 0x2000, None,
              0x4000, need, None) == -1           # no lse buffer
    assert al(C.byref(p), 4 * p.H, 0x1000, 0.1, C.byref(good), 0, 0x1000, C.byref(good), 0, 0x1000, 0x2000, 0x3002,
              0x4000, need, None) == -1           # misaligned lse buffer
    assert al(C.byref(p), 4 * p.H + 1, 0x1000, 0.1, C.byref(good), 0, 0x1000, C.byref(good), 0, 0x1000, 0x2000, 0x3000,
              0x4000, need, None) == -1
    assert wsb(C.byref(_params(D=32)), 4 * p.H) == 0 and wsb(C.byref(_params(D=64)), 4 * p.H) > 0
    assert lib.hqmq_last_hip_error() == 0


def test_build_codebooks_matches_the_oracles_generator(lib):
    for seed in (0, 1, 7, 42, 1337):
        mine = hq.hqmq_build_codebooks(seed, 3, 4, 48).numpy()
        ref = oracle.build_codebooks(seed, 3, 4, 48)
        ulp = np.abs(mine.view(np.int32).astype(np.int64) - ref.view(np.int32).astype(np.int64))
        assert ulp.max() <= 2
    # entry (layer, role, head, s) depends only on the seed and its linear index
    a = hq.hqmq_build_codebooks(5, 2, 4, 16)
    b = hq.hqmq_build_codebooks(5, 4, 4, 16)
    assert torch.equal(a, b[:2])
    assert np.abs(np.linalg.norm(a.numpy().astype(np.float64), axis=-1) - 1).max() < 1e-7
    with pytest.raises(hq.HqmqError):
        hq.hqmq_build_codebooks(0, 0, 4, 16)
    assert lib.hqmq_build_codebooks(0, 1, 1, 4, None) == -1
    buf = (C.c_float * 16)()
    assert lib.hqmq_build_codebooks(0, 1, 1, 3000, buf) == -2
    # one limit on S in every entry point: what the codebook call accepts, the encode takes
    big = (C.c_float * (2 * 4 * (hq.HQMQ_MAX_S + 1)))()   # [1 layer][2 roles][1 head][S][4]
    assert lib.hqmq_build_codebooks(0, 1, 1, hq.HQMQ_MAX_S, big) == 0
    assert lib.hqmq_build_codebooks(0, 1, 1, hq.HQMQ_MAX_S + 1, big) == -2
    hq.hqmq_sizes(_params(S=hq.HQMQ_MAX_S))
    with pytest.raises(hq.HqmqError):
        hq.hqmq_sizes(_params(S=hq.HQMQ_MAX_S + 1))
    header = open(os.path.join(ROOT, "include", "hqmq.h")).read()
    assert int(re.search(r"#define HQMQ_MAX_S (\d+)", header).group(1)) == hq.HQMQ_MAX_S
    assert "#define HQMQ_STATIC_SCRATCH_BYTES (16u << 20)" in header and hq.HQMQ_STATIC_SCRATCH_BYTES == 16 << 20


def test_host_entry_points_from_several_threads(lib):
    """The library keeps no state that distinct callers share (besides a per-device set-up flag): the
    host-side calls give every thread the same answers as a single thread, and the last-HIP-error word is
    per thread."""
    import threading
    want_info = hq.hqmq_sizes(_params())
    want_sec = hq.hqmq_build_codebooks(3, 1, 2, 24)
    errors = []

    def worker(seed):
        try:
            for i in range(200):
                info = hq.hqmq_sizes(_params())
                assert bytes(info) == bytes(want_info)
                good = binding._Encoded(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
                assert lib.hqmq_encode(C.byref(_params()), 0x1008, 0x1000, C.byref(good), 0, 0x1000,
                                       int(info.workspace_bytes), None) == -1
                if i % 50 == 0:
                    assert torch.equal(hq.hqmq_build_codebooks(3, 1, 2, 24), want_sec)
                assert lib.hqmq_last_hip_error() == 0
        except Exception as exc:       # noqa: BLE001 - reported by the main thread
            errors.append(exc)
    threads = [threading.Thread(target=worker, args=(k,)) for k in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_binding_refuses_host_tensors(lib):
    x = torch.zeros(1, 2, 4, 128, dtype=torch.float16)
    p = hq.params_for(x, 16)
    assert (p.stride_b, p.stride_h, p.stride_t) == (2 * 4 * 128, 4 * 128, 128)
    with pytest.raises(ValueError):
        hq.hqmq_encode(p, x, torch.zeros(2, 16, 4), None, None)
    with pytest.raises(ValueError):
        hq.params_for(x[..., ::2], 16)


def test_bench_refuses_more_than_one_gpu():
    """The measured path is single-GPU: bench.py --gpus N > 1 must say so and exit non-zero
    (checked before anything touches a GPU)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_division_by_the_biased_reciprocal_is_exact():
    """Decode and attention split a joint index into k / S and k mod S with uint(float(k) * inv_S),
    inv_S = fl(fl(1 / S) * (1 + 2^-18)) as the library's host code forms it: exact for every 16-bit k and
    every supported S (fp32 products as the GPU rounds them, conversion by truncation)."""
    k = np.arange(0, 65536, dtype=np.uint32)
    kf = k.astype(np.float32)
    for S in range(1, hq.HQMQ_MAX_S + 1):
        inv = np.float32(np.float32(1.0) / np.float32(S)) * np.float32(1.0 + 2.0 ** -18)
        assert np.array_equal((kf * np.float32(inv)).astype(np.uint32), k // S), S
