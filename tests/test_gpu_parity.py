"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle, element by
element, on seeded synthetic KV tensors.  Bit-exact on outlier masks, offsets, payload, scales
and radius codes; codeword indices identical outside near-ties (score gap < 1e-6), which are
counted; reconstruction within 1e-3 of the chunk norm."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_27646_amd as hq
import workloads
from gpu_util import (compare_decode, compare_encode, gpu_decode, gpu_encode, upload_encoded)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _bits(x: torch.Tensor) -> np.ndarray:
    return x.contiguous().cpu().numpy().view(np.uint16)


def _sec(seed, H, S, layer=0, role=0):
    cb = hq.hqmq_build_codebooks(seed, layer + 1, H, S)[layer, role].contiguous()
    return cb, cb.numpy()


def _roundtrip(x_cpu, S, b_r=6, Cmul=3.0, seed=0, rows=None, check_decode=True, flags=0):
    """Encode on both sides, compare; decode both encodings on both sides, compare."""
    B, H, T, D = x_cpu.shape
    sec_t, sec = _sec(seed, H, S)
    xb = _bits(x_cpu)
    e = oracle.encode(xb, sec, b_r=b_r, Cmul=Cmul, use_outliers=not (flags & hq.HQMQ_FLAG_NO_OUTLIERS),
                      rows=rows)
    x_dev, sec_dev = x_cpu.to(DEV), sec_t.to(DEV)
    g = gpu_encode(x_dev, sec_dev, b_r, Cmul, flags)
    stats = compare_encode(g, e, xb, sec)
    if check_decode:
        # (1) identical bytes, oracle-encoded (needs every row searched)
        if rows is None:
            want, r_hat = oracle.decode(e.codes, e.sigma, e.flags, e.row_off, e.outliers, sec, B, H, T, b_r, True, D=D)
            got = gpu_decode(g.params, upload_encoded(e, DEV), sec_dev, x_dev)
            stats["decode_rel_err_oracle_bytes"] = compare_decode(got, want, r_hat, e.flag)
        # (2) identical bytes, GPU-encoded
        want, r_hat = oracle.decode(g.codes, g.sigma, g.flags, g.row_off, g.outliers, sec, B, H, T, b_r, True, D=D)
        got = gpu_decode(g.params, g.bufs, sec_dev, x_dev)
        stats["decode_rel_err_gpu_bytes"] = compare_decode(got, want, r_hat, e.flag)
    print(stats, flush=True)
    return stats, e, g


def _lognormal_tensor(B, H, T, seed, sigma_g=0.5, D=128):
    wl = workloads.Workload("t", 100 + seed, 1, B, H, T, D, 16, sigma_g=sigma_g)
    return workloads.make_tensor(wl, 0, 0, "cpu")


# ---------------------------------------------------------------------------------------
# small shapes spanning several tiles and ragged tails
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("B,H,T,S,b_r", [
    (1, 1, 8, 16, 6),          # one partial block
    (1, 2, 333, 16, 6),        # ragged: not a multiple of 2, 8, 64 or 256 rows
    (2, 3, 77, 24, 4),         # batch > 1, S not a power of two (paper's s24_r4)
    (1, 8, 1024, 16, 6),       # the Tiny config shape
    (1, 2, 515, 64, 3),        # several scan blocks per segment, b_r = 3
    (1, 1, 130, 5, 6),         # S not a multiple of 4 (padded MFMA rows)
    (1, 1, 64, 1, 6),          # S = 1: the codebook is a rotated 24-cell
    (1, 1, 96, 192, 6),        # paper's s192_r6
    (1, 2, 150, 96, 4),        # paper's s96_r4
    (2, 1, 90, 48, 4),         # paper's s48_r4
    (1, 1, 70, 256, 6),        # S of the headline workload
    (1, 1, 40, 512, 8),        # largest S that is screened on the matrix cores, largest b_r
    (1, 2, 70, 600, 6),        # past it: every chunk scores all secondaries in fp32
    (2, 1, 20, 2730, 8),       # largest supported S (24 S = 65520) and b_r: 24-bit code words
    (1, 1, 300, 1024, 4),      # power of two above the screen's limit; 256-row workgroups
])
def test_encode_decode_parity_small(B, H, T, S, b_r):
    print(f"case B={B} H={H} T={T} S={S} b_r={b_r}", flush=True)
    x = _lognormal_tensor(B, H, T, seed=T + S, sigma_g=1.0)
    stats, e, g = _roundtrip(x, S, b_r)
    assert stats["outliers"] > 0 or T < 16


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        B = int(rng.integers(1, 4))
        H = int(rng.integers(1, 5))
        T = int(rng.integers(1, 160))
        S = int(rng.choice([1, 2, 3, 7, 16, 24, 33, 48, 64, 80]))
        b_r = int(rng.integers(1, 9))
        out.append((B, H, T, S, b_r))
    return out


@pytest.mark.parametrize("B,H,T,S,b_r", _random_shapes(14, seed=2024))
def test_encode_decode_parity_random_shapes(B, H, T, S, b_r):
    """Seeded random small shapes: every combination of batch, heads, ragged lengths, codebook sizes
    that are neither powers of two nor multiples of 16, and all radius widths."""
    x = _lognormal_tensor(B, H, T, seed=1000 + 7 * T + S, sigma_g=0.3 + 0.1 * b_r)
    _roundtrip(x, S, b_r=b_r, seed=S)


def test_tiny_config_full():
    wl = workloads.WORKLOADS["tiny"]
    for role in (0, 1):
        print(f"tiny role={role}", flush=True)
        x = workloads.make_tensor(wl, 0, role, "cpu")
        sec_t = hq.hqmq_build_codebooks(0, 1, wl.H, wl.S)[0, role].contiguous()
        sec = sec_t.numpy()
        xb = _bits(x)
        e = oracle.encode(xb, sec, b_r=wl.b_r, Cmul=wl.C)
        g = gpu_encode(x.to(DEV), sec_t.to(DEV), wl.b_r, wl.C)
        stats = compare_encode(g, e, xb, sec)
        print(stats, flush=True)
        assert 0.003 < stats["outliers"] / e.flag.size < 0.03


@pytest.mark.parametrize("name", ["mistral7b_outlier", "qwen25_7b_heavy", "llama3_70b_128k"])
def test_outlier_heavy_laws_reduced_length(name):
    """The hot-channel / heavy-tailed / wide-lognormal value laws at a reduced sequence length
    (the full-size shapes are covered by the sampled test below)."""
    wl = workloads.WORKLOADS[name].with_T(700 if name != "mistral7b_outlier" else 200)
    print(f"law {name} T={wl.T}", flush=True)
    x = workloads.make_tensor(wl, 0, 0, "cpu")
    stats, e, g = _roundtrip(x, wl.S, wl.b_r)
    assert stats["outliers"] / e.flag.size > 0.01


# ---------------------------------------------------------------------------------------
# full-size tensor in the launch configuration the bench times
# ---------------------------------------------------------------------------------------

def test_llama3_8b_32k_layer_every_row():
    """One full [1, 8, 32768, 128] tensor with S = 256, every step on every row: norms, medians, masks,
    offsets, payload, scales, radius codes, the exhaustive search of all 8.4 M chunks, and the decode of
    both sides' bytes (the oracle takes about 20 s on 16 threads)."""
    wl = workloads.WORKLOADS["llama3_8b_32k"]
    x = workloads.make_tensor(wl, 3, 0, "cpu")
    stats, e, g = _roundtrip(x, wl.S, wl.b_r, check_decode=True)
    assert 0.005 < stats["outliers"] / e.flag.size < 0.03
    assert stats["near_ties"] < 1e-3 * stats["chunks"]


def test_llama3_8b_32k_in_the_bench_launch_configuration():
    """The launches bench.py times: 32 full-size tensors per hqmq_encode_batch / hqmq_decode_batch
    launch.  One of them (slot 21 = layer 10, V) is checked against the oracle like the single-tensor
    test above (O(n) steps on all rows, the search on sampled rows, decode of the GPU's bytes); every
    tensor of the launch must carry its own, not a neighbour's, data: slot 4 is compared with a
    single-tensor encode of the same input."""
    wl = workloads.WORKLOADS["llama3_8b_32k"]
    n = 32
    cb = hq.hqmq_build_codebooks(0, n // 2, wl.H, wl.S)
    slot = 21
    x_cpu = workloads.make_tensor(wl, slot // 2, slot % 2, "cpu")
    xs, secs = [], []
    for i in range(n):
        xs.append(x_cpu.to(DEV) if i == slot else workloads.make_tensor(wl, i // 2, i % 2, DEV))
        secs.append(cb[i // 2, i % 2].contiguous().to(DEV))
    params = hq.params_for(xs[0], wl.S, wl.b_r, wl.C)
    encs = [hq.alloc_encoded(params, DEV) for _ in range(n)]
    ws = hq.alloc_batch_workspace(params, n, DEV)
    ws.fill_(0xAB)
    hq.hqmq_encode_batch(hq.EncodeBatch(params, xs, secs, encs, ws))
    outs = [torch.full_like(x, float("nan")) for x in xs]
    hq.hqmq_decode_batch(hq.DecodeBatch(params, encs, secs, outs))
    torch.cuda.synchronize()

    # slot 4 against a single-tensor call
    single = gpu_encode(xs[4], secs[4], wl.b_r, wl.C)
    assert torch.equal(encs[4].codes, single.bufs.codes) and torch.equal(encs[4].flags, single.bufs.flags)
    assert torch.equal(encs[4].row_off, single.bufs.row_off) and torch.equal(encs[4].n_outliers, single.bufs.n_outliers)
    assert np.array_equal(outs[4].cpu().numpy().view(np.uint16), gpu_decode(params, single.bufs, secs[4], xs[4]))

    # slot 21 against the oracle
    from gpu_util import GpuEncoded
    b = encs[slot]
    n_out = b.n_outliers.cpu().numpy().view(np.uint32)
    total = int(n_out[-1])
    g = GpuEncoded(params, b, b.codes.cpu().numpy().view(np.uint32), b.sigma.cpu().numpy().view(np.uint16),
                   b.flags.cpu().numpy().view(np.uint32), b.row_off.cpu().numpy().view(np.uint32), n_out,
                   b.outliers[:total].cpu().numpy().view(np.uint16).reshape(total, 4),
                   int(b.status.cpu().numpy().view(np.uint32)[0]))
    sec = cb[slot // 2, slot % 2].numpy()
    xb = _bits(x_cpu)
    rows = workloads.sample_rows(wl, 32, 32, 96, seed=5).numpy()
    e = oracle.encode(xb, sec, b_r=wl.b_r, Cmul=wl.C, rows=rows)
    stats = compare_encode(g, e, xb, sec)
    want, r_hat = oracle.decode(g.codes, g.sigma, g.flags, g.row_off, g.outliers, sec, wl.B, wl.H, wl.T, wl.b_r, True)
    stats["decode_rel_err"] = compare_decode(outs[slot].cpu().numpy().view(np.uint16), want, r_hat, e.flag)
    print(stats, flush=True)


@pytest.mark.parametrize("name,layer,role", [
    ("mha32_d96_8k", 3, 0),          # [1, 32, 8192, 96], S = 192, b_r = 4: 24 chunks per row
    ("gqa8_d64_32k", 1, 0),          # [1, 8, 32768, 64], S = 192, b_r = 4: 16 chunks per row, hot channels
    ("mistral7b_outlier", 5, 0),     # [4, 8, 8192, 128], S = 64: batch > 1, hot channels (about 10 % outliers)
    ("qwen25_7b_heavy", 2, 0),       # [1, 4, 32768, 128], S = 256: hot channels + heavy-tailed spikes
    ("llama3_70b_128k", 7, 1),       # [1, 8, 131072, 128], S = 256: 256 MiB per tensor, four times the rows
])
def test_other_workloads_full_size(name, layer, role):
    """One full-size tensor of each remaining workload, as the library is launched on it: every step on
    every row (about 10 s of oracle time each), except for the 128k-token tensor, whose search is compared
    on a sample of token rows of every head (all its O(n) results, and its decode, still on every row)."""
    wl = workloads.WORKLOADS[name]
    x = workloads.make_tensor(wl, layer, role, "cpu")
    rows = None if name != "llama3_70b_128k" else workloads.sample_rows(wl, 16, 16, 64, seed=2).numpy()
    print(f"{name} layer {layer} role {role}: searching "
          f"{'all' if rows is None else int(rows.sum())} of {wl.B * wl.H * wl.T} rows on the CPU", flush=True)
    stats, e, g = _roundtrip(x, wl.S, wl.b_r, rows=rows, check_decode=(name != "llama3_70b_128k"))
    assert stats["near_ties"] < 1e-3 * stats["chunks"]
    if name == "llama3_70b_128k":
        # decode parity on every row: both decoders on the GPU-encoded bytes (the oracle's own encoding has
        # codes on the sampled rows only)
        want, r_hat = oracle.decode(g.codes, g.sigma, g.flags, g.row_off, g.outliers, _sec(0, wl.H, wl.S)[1],
                                    wl.B, wl.H, wl.T, wl.b_r, True)
        got = gpu_decode(g.params, g.bufs, _sec(0, wl.H, wl.S)[0].to(DEV), x.to(DEV))
        compare_decode(got, want, r_hat, e.flag)


# ---------------------------------------------------------------------------------------
# head dimensions other than 128 (the paper's models: 64, 96, 128; anything else through zero padding)
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("D,B,H,T,S,b_r", [
    (64, 1, 2, 333, 16, 6),      # 16 chunks per row, ragged length
    (64, 2, 3, 77, 24, 4),       # the paper's s24_r4
    (96, 1, 2, 515, 192, 4),     # 24 chunks per row, the paper's s192_r4; several scan blocks
    (96, 2, 1, 64, 48, 3),
    (32, 1, 4, 130, 5, 6),
    (4, 1, 1, 300, 16, 6),       # one chunk per row
    (45, 1, 2, 200, 24, 4),      # the paper's padding example: 12 chunks, the last one holds 1 element
    (1, 1, 1, 70, 16, 6),        # one element per row
    (100, 2, 2, 90, 33, 5),      # multiple of 4, strides not multiples of 8
    (126, 1, 1, 130, 256, 6),    # 32 chunks like the full row, but through the general path
    (124, 1, 3, 2100, 64, 6),    # 31 chunks; long enough for the 256-row search workgroups
    (96, 1, 1, 2100, 256, 6),    # long, but the tables leave no room for 256-row workgroups: 8 waves, 64 rows
    (96, 1, 1, 70, 512, 8),      # largest S and b_r at 24 chunks per row
    (124, 1, 1, 70, 512, 8),     # the most LDS the general search can ask for
    (96, 1, 2, 40, 700, 6),      # unscreened search at 24 chunks per row
    (64, 1, 1, 30, 2730, 8),     # largest S at 16 chunks per row
    (64, 1, 2, 4100, 192, 4),    # 256-row workgroups at 16 chunks per row, ragged last workgroup
])
def test_other_head_dimensions_small(D, B, H, T, S, b_r):
    print(f"case D={D} B={B} H={H} T={T} S={S} b_r={b_r}", flush=True)
    x = _lognormal_tensor(B, H, T, seed=D + T, sigma_g=1.0, D=D)
    stats, e, g = _roundtrip(x, S, b_r)
    info = hq.hqmq_sizes(g.params)
    nc = -(-D // 4)
    assert info.chunks_per_row == nc and info.code_words_per_row == -(-nc * info.code_bits // 32)
    assert stats["outliers"] > 0


@pytest.mark.parametrize("D,pitch", [(45, 53), (96, 104), (64, 64 + 8), (3, 4)])
def test_other_head_dimensions_touch_nothing_past_the_row(D, pitch):
    """Rows stored with a pitch larger than D: encode must not read, and decode must not write, the
    elements between D and the pitch (encode: the gap holds huge values that would change every
    median, scale and flag; decode: the gap keeps its sentinel)."""
    B, H, T, S, b_r = 2, 2, 61, 24, 4
    x = _lognormal_tensor(B, H, T, seed=D, sigma_g=1.0, D=D)
    sec_t, sec = _sec(1, H, S)
    e = oracle.encode(_bits(x), sec, b_r=b_r)
    wide = torch.full((B, H, T, pitch), 60000.0, dtype=torch.float16, device=DEV)
    wide[..., :D] = x.to(DEV)
    view = wide[..., :D]
    assert view.stride(2) == pitch
    g = gpu_encode(view, sec_t.to(DEV), b_r)
    compare_encode(g, e, _bits(x), sec)
    out_wide = torch.full((B, H, T, pitch), -7.0, dtype=torch.float16, device=DEV)
    out = out_wide[..., :D]
    hq.hqmq_decode(hq.params_for(out, S, b_r), g.bufs, sec_t.to(DEV), out)
    torch.cuda.synchronize()
    assert bool((out_wide[..., D:] == -7.0).all())
    want, r_hat = oracle.decode(g.codes, g.sigma, g.flags, g.row_off, g.outliers, sec, B, H, T, b_r, True, D=D)
    compare_decode(out.contiguous().cpu().numpy().view(np.uint16), want, r_hat, e.flag)


def test_other_head_dimensions_batched_and_incremental():
    """D = 96: a batch of tensors in one launch equals the single calls, and appended token rows
    encode against thresholds taken from the prefill."""
    B, H, T, S, b_r, D, n = 1, 3, 140, 48, 4, 96, 3
    sec_t, sec = _sec(2, H, S)
    sec_dev = sec_t.to(DEV)
    xs = [_lognormal_tensor(B, H, T, seed=300 + i, sigma_g=0.8, D=D) for i in range(n)]
    xd = [x.to(DEV) for x in xs]
    params = hq.params_for(xd[0], S, b_r)
    encs = [hq.alloc_encoded(params, DEV) for _ in range(n)]
    ws = hq.alloc_batch_workspace(params, n, DEV)
    hq.hqmq_encode_batch(hq.EncodeBatch(params, xd, [sec_dev] * n, encs, ws))
    thr = hq.hqmq_thresholds(params, ws, 1)
    torch.cuda.synchronize()
    for i in range(n):
        e = oracle.encode(_bits(xs[i]), sec, b_r=b_r)
        bufs = encs[i]
        n_out = bufs.n_outliers.cpu().numpy().view(np.uint32)
        total = int(n_out[-1])
        from gpu_util import GpuEncoded
        g = GpuEncoded(params, bufs, bufs.codes.cpu().numpy().view(np.uint32), bufs.sigma.cpu().numpy().view(np.uint16),
                       bufs.flags.cpu().numpy().view(np.uint32), bufs.row_off.cpu().numpy().view(np.uint32), n_out,
                       bufs.outliers[:total].cpu().numpy().view(np.uint16).reshape(total, 4),
                       int(bufs.status.cpu().numpy().view(np.uint32)[0]))
        compare_encode(g, e, _bits(xs[i]), sec)
        if i == 1:
            assert np.array_equal(thr.cpu().numpy(), 9.0 * e.m2)
    new = (_lognormal_tensor(B, H, 2, seed=400, sigma_g=0.8, D=D) * 1.7).to(torch.float16)
    e = oracle.encode(_bits(new), sec, b_r=b_r, thresholds=thr.cpu().numpy())
    p2 = hq.params_for(new.to(DEV), S, b_r)
    bufs = hq.alloc_encoded(p2, DEV, outlier_capacity=B * H * 2 * 24)
    hq.hqmq_encode_given_thresholds(p2, new.to(DEV), sec_dev, thr, bufs, hq.alloc_workspace(p2, DEV))
    torch.cuda.synchronize()
    n_out = bufs.n_outliers.cpu().numpy().view(np.uint32)
    total = int(n_out[-1])
    g = GpuEncoded(p2, bufs, bufs.codes.cpu().numpy().view(np.uint32), bufs.sigma.cpu().numpy().view(np.uint16),
                   bufs.flags.cpu().numpy().view(np.uint32), bufs.row_off.cpu().numpy().view(np.uint32), n_out,
                   bufs.outliers[:total].cpu().numpy().view(np.uint16).reshape(total, 4),
                   int(bufs.status.cpu().numpy().view(np.uint32)[0]))
    compare_encode(g, e, _bits(new), sec)


# ---------------------------------------------------------------------------------------
# a cache whose token axis is split over shards: the median is found by exchanging histograms
# ---------------------------------------------------------------------------------------

def _sharded_thresholds(shards_dev, S, b_r, Cmul):
    """Run the 6 counting passes and the finish on every shard; between passes sum the pass's histogram
    over the shards and write it back to each (what an all-reduce would do).  Returns thresholds per shard."""
    ps = [hq.params_for(x, S, b_r, Cmul) for x in shards_dev]
    wss = [hq.alloc_workspace(p, DEV) for p in ps]
    for ws in wss:
        ws.fill_(0xCD)
    total = sum(p.B * p.T * (-(-p.D // 4)) for p in ps)
    for pas in range(6):
        for p, x, ws in zip(ps, shards_dev, wss):
            hq.hqmq_shard_median_pass(p, total, pas, x, ws)
        regions = [hq.hqmq_shard_median_region(p, pas, ws) for p, ws in zip(ps, wss)]
        summed = torch.stack(regions).sum(0, dtype=torch.int32)
        assert int(summed.sum()) <= total * ps[0].H
        for r in regions:
            r.copy_(summed)
    out = []
    for p, x, ws in zip(ps, shards_dev, wss):
        hq.hqmq_shard_median_pass(p, total, 6, x, ws)
        out.append(hq.hqmq_thresholds(p, ws))
    torch.cuda.synchronize()
    return ps, out


@pytest.mark.parametrize("D,splits,kind", [
    (128, (700, 1, 323), "lognormal"),      # ragged shards, one of a single token
    (96, (256, 300), "lognormal"),
    (128, (128, 128, 128, 128), "equal"),   # every norm equal: all keys fall into one bin in every pass
    (64, (50, 77), "few_values"),           # coarsely quantised data: heavy ties around the median
])
def test_sequence_sharded_median_and_encode(D, splits, kind):
    B, H, S, b_r, Cmul = 2, 3, 24, 4, 3.0
    T = sum(splits)
    x = _lognormal_tensor(B, H, T, seed=77 + D, sigma_g=0.9, D=D)
    if kind == "equal":
        x = torch.full_like(x, 0.5)
    elif kind == "few_values":
        x = (x * 2).round().clamp(-3, 3).to(torch.float16) / 2
    sec_t, sec = _sec(4, H, S)
    whole = oracle.encode(_bits(x), sec, b_r=b_r, Cmul=Cmul, rows=np.zeros(B * H * T, bool))
    want_thr = np.float64(np.float32(Cmul)) ** 2 * whole.m2
    bounds = np.cumsum((0,) + splits)
    shards = [x[:, :, a:b].contiguous() for a, b in zip(bounds[:-1], bounds[1:])]
    shards_dev = [s.to(DEV) for s in shards]
    ps, thrs = _sharded_thresholds(shards_dev, S, b_r, Cmul)
    for t in thrs:
        assert np.array_equal(t.cpu().numpy(), want_thr)       # bit-exact, and the same on every shard
    # every shard encodes its slice against the common thresholds: equal to the oracle on that slice,
    # and the flags are those of the unsharded tensor
    fl_whole = whole.flag.reshape(B, H, T, -1)
    sec_dev = sec_t.to(DEV)
    from gpu_util import GpuEncoded
    for (a, b), sh, shd, p in zip(zip(bounds[:-1], bounds[1:]), shards, shards_dev, ps):
        e = oracle.encode(_bits(sh), sec, b_r=b_r, thresholds=want_thr)
        assert np.array_equal(e.flag.reshape(B, H, b - a, -1), fl_whole[:, :, a:b])
        nc = e.r2.shape[1]
        bufs = hq.alloc_encoded(p, DEV, outlier_capacity=B * H * (b - a) * nc)
        hq.hqmq_encode_given_thresholds(p, shd, sec_dev, thrs[0], bufs, hq.alloc_workspace(p, DEV))
        torch.cuda.synchronize()
        n_out = bufs.n_outliers.cpu().numpy().view(np.uint32)
        total = int(n_out[-1])
        g = GpuEncoded(p, bufs, bufs.codes.cpu().numpy().view(np.uint32), bufs.sigma.cpu().numpy().view(np.uint16),
                       bufs.flags.cpu().numpy().view(np.uint32), bufs.row_off.cpu().numpy().view(np.uint32), n_out,
                       bufs.outliers[:total].cpu().numpy().view(np.uint16).reshape(total, 4),
                       int(bufs.status.cpu().numpy().view(np.uint32)[0]))
        compare_encode(g, e, _bits(sh), sec)


def test_sequence_sharded_median_equals_the_single_call_select():
    """One shard holding everything: the histogram-only select and the encode's own select agree."""
    x = _lognormal_tensor(1, 4, 3000, seed=91, sigma_g=0.7)
    sec_t, _ = _sec(0, 4, 16)
    xd = x.to(DEV)
    ps, thrs = _sharded_thresholds([xd], 16, 6, 3.0)
    ws = hq.alloc_workspace(ps[0], DEV)
    hq.hqmq_encode(ps[0], xd, sec_t.to(DEV), hq.alloc_encoded(ps[0], DEV), ws)
    assert torch.equal(hq.hqmq_thresholds(ps[0], ws), thrs[0])


# ---------------------------------------------------------------------------------------
# degenerate inputs and the boundary's data-dependent behaviour
# ---------------------------------------------------------------------------------------

def test_single_token_row():
    x = _lognormal_tensor(1, 2, 1, seed=5)
    _roundtrip(x, 16)


def test_all_zero_and_constant_tensors():
    z = torch.zeros(1, 2, 40, 128, dtype=torch.float16)
    stats, e, g = _roundtrip(z, 16)
    assert stats["outliers"] == 0 and not g.codes.any() and not g.sigma.any()
    c = torch.full((1, 2, 40, 128), 0.5, dtype=torch.float16)
    stats, e, g = _roundtrip(c, 16)
    assert stats["outliers"] == 0                      # equal norms: nothing exceeds 3x the median
    half = torch.zeros(1, 1, 64, 128, dtype=torch.float16)
    half[:, :, :, :40] = 1.0                            # median norm 0: every non-zero chunk is flagged
    stats, e, g = _roundtrip(half, 16)
    assert stats["outliers"] == 64 * 10


def test_median_with_many_equal_norms():
    """More equal chunk norms than the select kernel's candidate list holds (16384 per head):
    the exact median must still come out (slow path that re-reads the head's rows)."""
    x = torch.ones(1, 2, 1100, 128, dtype=torch.float16)             # 35200 chunks of norm 2 per head
    x[0, 0, :300] = 3.0                                               # head 0: 9600 larger ...
    x[0, 0, 300:320, :64] = 40.0                                      # ... and a few outliers
    x[0, 1, ::2] = 2.0                                                # head 1: two values, half each
    x[0, 1, 7, 4:8] = 9.0
    stats, e, g = _roundtrip(x, 16)
    assert stats["outliers"] == 20 * 16 + 1


@pytest.mark.parametrize("spread", [0.004, 0.03, 0.2])
def test_median_of_concentrated_norms(spread):
    """Norms packed into a narrow band: the bin of the select's first digit that holds the median then
    holds from a few per cent to most of a head's chunks, more than a workgroup stages (0.03) and more
    than the candidate list keeps (0.004: the third sweep has to narrow it down).  Thresholds bit for
    bit, and with them every flag word."""
    B, H, T, S = 1, 2, 4096, 1
    gen = torch.Generator().manual_seed(int(spread * 1e4))
    mag = 1.0 + spread * (2.0 * torch.rand(B, H, T, 128, generator=gen) - 1.0)
    sign = torch.where(torch.rand(B, H, T, 128, generator=gen) < 0.5, -1.0, 1.0)
    x = (mag * sign).half()
    x[0, 1] *= 37.0                                        # the second head in another binade
    x[0, :, ::7, :4] *= 6.0                                # some outliers
    sec_t, sec = _sec(4, H, S)
    xb = _bits(x)
    e = oracle.encode(xb, sec, rows=np.arange(0, B * H * T, 97))
    x_dev, sec_dev = x.to(DEV), sec_t.to(DEV)
    g = gpu_encode(x_dev, sec_dev)
    stats = compare_encode(g, e, xb, sec)
    print(stats, flush=True)
    params = hq.params_for(x_dev, S)
    ws = hq.alloc_workspace(params, DEV)
    hq.hqmq_encode(params, x_dev, sec_dev, hq.alloc_encoded(params, DEV), ws)
    thr = hq.hqmq_thresholds(params, ws)
    torch.cuda.synchronize()
    c = float(np.float32(3.0))
    assert np.array_equal(thr.cpu().numpy().view(np.uint64), ((c * c) * e.m2).view(np.uint64))
    assert stats["outliers"] > 0


def test_sampled_select_and_its_fallbacks():
    """Heads of at least 2^17 chunks: the select predicts the median's bin from every 16th row.  One head
    whose sample is representative, one whose sampled rows are eight times smaller than the rest (the
    prediction misses and the bin is collected by a sweep of its own), one of equal norms (every list
    overflows: the slow exact path), one of zeros, and one whose sampled rows alone are zero.
    Thresholds bit for bit."""
    B, H, T, S = 1, 5, 8192, 1
    gen = torch.Generator().manual_seed(77)
    x = torch.randn(B, H, T, 128, generator=gen) * torch.exp(0.5 * torch.randn(B, H, T, 1, generator=gen))
    x[0, 1, ::16] *= 0.125
    x[0, 2] = 0.75
    x[0, 3] = 0.0
    x[0, 4, ::16] = 0.0
    x = x.half()
    sec_t, sec = _sec(4, H, S)
    xb = _bits(x)
    e = oracle.encode(xb, sec, rows=np.arange(0, B * H * T, 211))
    x_dev, sec_dev = x.to(DEV), sec_t.to(DEV)
    g = gpu_encode(x_dev, sec_dev)
    stats = compare_encode(g, e, xb, sec)
    print(stats, flush=True)
    params = hq.params_for(x_dev, S)
    ws = hq.alloc_workspace(params, DEV)
    hq.hqmq_encode(params, x_dev, sec_dev, hq.alloc_encoded(params, DEV), ws)
    thr = hq.hqmq_thresholds(params, ws)
    torch.cuda.synchronize()
    c = float(np.float32(3.0))
    assert np.array_equal(thr.cpu().numpy().view(np.uint64), ((c * c) * e.m2).view(np.uint64))
    assert e.m2[3] == 0.0 and e.m2[2] == 4 * 0.75 ** 2


@pytest.mark.parametrize("kind,D,B,H,T", [
    ("plain", 128, 1, 2, 9000), ("ramp", 96, 2, 2, 4000), ("sampled rows small", 64, 1, 3, 12000),
    ("sampled rows large", 128, 2, 1, 5000), ("narrow band", 96, 1, 2, 6000), ("half the rows zero", 128, 1, 2, 8200),
    ("coarse values", 64, 2, 2, 7000),
])
def test_sampled_select_row_structures(kind, D, B, H, T):
    """Heads of 2^17 chunks and more whose rows are not drawn from one distribution, in ways that mislead the
    every-16th-row sample or overflow the candidate list: thresholds bit for bit, encode on sampled rows."""
    gen = torch.Generator().manual_seed(len(kind) * 1000 + T)
    x = torch.randn(B, H, T, D, generator=gen) * torch.exp(0.6 * torch.randn(B, H, T, 1, generator=gen))
    t = torch.arange(T).view(1, 1, T, 1)
    if kind == "ramp":
        x = x * (0.2 + 3.0 * t / T)
    elif kind == "sampled rows small":
        x = x * torch.where(t % 16 == 0, 0.05, 1.0)
    elif kind == "sampled rows large":
        x = x * torch.where(t % 16 == 0, 30.0, 1.0)
    elif kind == "narrow band":
        x = (1.0 + 0.003 * torch.randn(B, H, T, D, generator=gen)) * torch.where(
            torch.rand(B, H, T, D, generator=gen) < 0.5, -1.0, 1.0)
    elif kind == "half the rows zero":
        x = x * torch.where(t < T // 2, 0.0, 1.0)
    elif kind == "coarse values":
        x = torch.round(x * 2) / 2
    x = x.half()
    S = 1
    sec_t, sec = _sec(4, H, S)
    xb = _bits(x)
    e = oracle.encode(xb, sec, rows=np.arange(0, B * H * T, 499))
    x_dev, sec_dev = x.to(DEV), sec_t.to(DEV)
    g = gpu_encode(x_dev, sec_dev)
    print(compare_encode(g, e, xb, sec), flush=True)
    params = hq.params_for(x_dev, S)
    ws = hq.alloc_workspace(params, DEV)
    hq.hqmq_encode(params, x_dev, sec_dev, hq.alloc_encoded(params, DEV), ws)
    thr = hq.hqmq_thresholds(params, ws)
    torch.cuda.synchronize()
    c = float(np.float32(3.0))
    assert np.array_equal(thr.cpu().numpy().view(np.uint64), ((c * c) * e.m2).view(np.uint64))


def test_exact_tie_structured_input():
    """Chunks like (a, a, 0, 0) sit on the boundary between several codewords when the
    secondary is the identity; whichever the GPU picks must score as the oracle's best."""
    x = torch.zeros(1, 1, 16, 128, dtype=torch.float16)
    x[..., 0::4] = 1.0
    x[..., 1::4] = 1.0
    sec = np.array([[[1, 0, 0, 0]]], np.float32)
    xb = _bits(x)
    e = oracle.encode(xb, sec)
    g = gpu_encode(x.to(DEV), torch.from_numpy(sec).to(DEV))
    stats = compare_encode(g, e, xb, sec)
    k, _ = oracle.unpack_rows(g.codes, 1, 6)
    assert (k == 0).all()                               # lowest index of the six tied vertices
    assert stats["near_ties"] == 16 * 32


@pytest.mark.parametrize("S,pairs", [(80, [(2, 19), (7, 40), (33, 79), (64, 65)]), (5, [(1, 4)]), (256, [(0, 255), (100, 101)])])
def test_codebook_with_repeated_secondaries(S, pairs):
    """Two bit-identical secondaries score identically for every chunk, whatever group of the matrix
    pass they sit in: the library has to notice that the two groups cannot be told apart, search the
    chunk again with plain fp32 arithmetic, and return the lower index like the oracle."""
    x = _lognormal_tensor(1, 1, 96, seed=31 + S, sigma_g=0.7)
    sec = _sec(3, 1, S)[1].copy()
    for lo, hi in pairs:
        sec[0, hi] = sec[0, lo]
    xb = _bits(x)
    e = oracle.encode(xb, sec, b_r=6, Cmul=3.0)
    g = gpu_encode(x.to(DEV), torch.from_numpy(sec).to(DEV), 6, 3.0)
    stats = compare_encode(g, e, xb, sec)
    print(stats, flush=True)
    assert stats["near_ties"] >= 10 * len(pairs) // 2       # the chunks nearest to a repeated secondary
    assert stats["index_mismatch_in_near_ties"] == 0
    k, _ = oracle.unpack_rows(g.codes, S, 6)
    assert not np.isin(k % S, [hi for _, hi in pairs]).any()  # never the second copy


def test_codebook_with_nearly_equal_secondaries():
    """Secondaries that differ in their last bits only: scores closer than the matrix pass resolves.
    Whichever codeword the library returns must score within 1e-6 of the oracle's best."""
    S = 112
    x = _lognormal_tensor(1, 2, 128, seed=77, sigma_g=0.7)
    sec = _sec(5, 2, S)[1].copy()
    rng = np.random.default_rng(5)
    for lo, hi in [(3, 50), (20, 111), (21, 22), (64, 9)]:
        sec[:, hi] = sec[:, lo] * (1.0 + rng.uniform(-2e-7, 2e-7, size=(2, 4))).astype(np.float32)
    xb = _bits(x)
    e = oracle.encode(xb, sec, b_r=4, Cmul=3.0)
    g = gpu_encode(x.to(DEV), torch.from_numpy(sec).to(DEV), 4, 3.0)
    stats = compare_encode(g, e, xb, sec)
    print(stats, flush=True)
    assert stats["near_ties"] > 100


def test_direction_component_on_a_half_precision_midpoint():
    """Regression: the matrix pass splits every direction component into two fp16 parts; both must be
    taken from the same fp32 value.  Row 630 of this tensor holds a chunk whose fourth component, scaled, is
    exactly halfway between two fp16 values; a build whose two conversions rounded it differently ranked
    the runner-up codeword (6e-5 behind) first."""
    x = _lognormal_tensor(2, 3, 4096, seed=582616, sigma_g=0.7)
    stats, e, g = _roundtrip(x, 3, b_r=4, Cmul=1.5, seed=60, check_decode=False)
    # the chunk in question has a gap of 6e-5, far from a near-tie: the comparison inside _roundtrip
    # rejects any index that differs at such a gap; what is left may only differ inside near-ties
    k_gpu, _ = oracle.unpack_rows(g.codes, 3, 4, 32)
    differs = (e.flag == 0) & (k_gpu != e.k)
    assert not (differs & ((e.best - e.second) >= 1e-6)).any()
    assert int(differs.sum()) == stats["index_mismatch_in_near_ties"] <= stats["near_ties"]


def test_extreme_magnitudes():
    x = _lognormal_tensor(1, 2, 64, seed=9).float()
    x[0, 0, :8] *= 6e-6                                 # subnormal fp16 territory
    x[0, 1, :8] = x[0, 1, :8].sign() * 65504.0          # largest finite halves: sigma saturates
    x[0, 1, 8:16] *= 3000.0
    _roundtrip(x.clamp(-65504, 65504).half(), 16)


def test_no_outliers_flag():
    x = _lognormal_tensor(1, 2, 100, seed=11, sigma_g=1.5)
    stats, e, g = _roundtrip(x, 16, flags=hq.HQMQ_FLAG_NO_OUTLIERS)
    assert stats["outliers"] == 0 and not g.flags.any()


def test_other_multiplier():
    x = _lognormal_tensor(1, 2, 128, seed=12)
    stats, _, _ = _roundtrip(x, 16, Cmul=1.5)
    assert stats["outliers"] > 100


def test_outlier_overflow_reports_true_counts():
    x = _lognormal_tensor(1, 2, 256, seed=13, sigma_g=1.0)
    sec_t, sec = _sec(0, 2, 16)
    xb = _bits(x)
    e = oracle.encode(xb, sec)
    total = int(e.n_out[-1])
    assert total > 10
    g = gpu_encode(x.to(DEV), sec_t.to(DEV), outlier_capacity=total // 2)
    assert g.status & hq.HQMQ_STATUS_OUTLIER_OVERFLOW
    assert np.array_equal(g.n_out, e.n_out) and np.array_equal(g.row_off, e.row_off)
    assert np.array_equal(g.outliers, e.outliers[: total // 2])       # the prefix that fits is right
    # decoding the truncated encoding stays in bounds: dropped outliers come back as zeros
    out = gpu_decode(g.params, g.bufs, sec_t.to(DEV), x.to(DEV)).reshape(-1, 32, 4)
    fl = e.flag.astype(bool)
    pos = np.cumsum(fl.reshape(-1)).reshape(fl.shape) - 1
    assert not out[fl & (pos >= total // 2)].any()
    exact = gpu_encode(x.to(DEV), sec_t.to(DEV), outlier_capacity=total)
    assert exact.status == 0 and np.array_equal(exact.outliers, e.outliers)


def test_strided_input_and_output():
    """A cache stored [B, T, H, D] passes unchanged through the strides."""
    B, H, T = 2, 3, 50
    x = _lognormal_tensor(B, H, T, seed=14)
    sec_t, sec = _sec(0, H, 16)
    e = oracle.encode(_bits(x), sec)
    x_bthd = x.permute(0, 2, 1, 3).contiguous().to(DEV)           # memory order [B, T, H, D]
    view = x_bthd.permute(0, 2, 1, 3)                               # logical [B, H, T, D]
    assert not view.is_contiguous()
    g = gpu_encode(view, sec_t.to(DEV))
    compare_encode(g, e, _bits(x), sec)
    out = torch.zeros_like(x_bthd).permute(0, 2, 1, 3)
    hq.hqmq_decode(hq.params_for(out, 16), g.bufs, sec_t.to(DEV), out)
    torch.cuda.synchronize()
    want, r_hat = oracle.decode(g.codes, g.sigma, g.flags, g.row_off, g.outliers, sec, B, H, T, 6, True)
    compare_decode(out.contiguous().cpu().numpy().view(np.uint16), want, r_hat, e.flag)


@pytest.mark.parametrize("D", [128, 96])
def test_strided_input_long_enough_for_the_sampled_select(D):
    """[B, T, H, D] memory order with heads of more than 2^17 chunks (the select reads every 16th row first)
    and a pitch above D: thresholds bit for bit, encode on sampled rows."""
    B, H, T, S = 2, 2, 3000 if D == 128 else 4000, 8
    x = _lognormal_tensor(B, H, T, seed=31, D=D)
    sec_t, sec = _sec(2, H, S)
    xb = _bits(x)
    e = oracle.encode(xb, sec, rows=np.arange(0, B * H * T, 53))
    store = torch.zeros(B, T, H, D + 8, dtype=torch.float16)
    store[..., :D] = x.permute(0, 2, 1, 3)
    view = store.to(DEV).permute(0, 2, 1, 3)[..., :D]              # logical [B, H, T, D], pitch D + 8
    assert not view.is_contiguous()
    g = gpu_encode(view, sec_t.to(DEV))
    stats = compare_encode(g, e, xb, sec)
    print(stats, flush=True)
    params = hq.params_for(view, S)
    ws = hq.alloc_workspace(params, DEV)
    hq.hqmq_encode(params, view, sec_t.to(DEV), hq.alloc_encoded(params, DEV), ws)
    thr = hq.hqmq_thresholds(params, ws)
    torch.cuda.synchronize()
    c = float(np.float32(3.0))
    assert np.array_equal(thr.cpu().numpy().view(np.uint64), ((c * c) * e.m2).view(np.uint64))


def test_decode_batch_equals_single_decodes():
    """One launch for many tensors of a shape must give each tensor exactly hqmq_decode's bytes
    (40 tensors: more than one launch's worth of descriptors)."""
    B, H, T, S = 1, 2, 70, 16
    n = 40
    cb = hq.hqmq_build_codebooks(3, n, H, S)
    xs, encs, secs, singles = [], [], [], []
    for i in range(n):
        x = _lognormal_tensor(B, H, T, seed=200 + i, sigma_g=1.0).to(DEV)
        sec = cb[i, i % 2].contiguous().to(DEV)
        g = gpu_encode(x, sec)
        xs.append(x)
        encs.append(g.bufs)
        secs.append(sec)
        singles.append(gpu_decode(g.params, g.bufs, sec, x))
    params = hq.params_for(xs[0], S)
    outs = [torch.full_like(x, float("nan")) for x in xs]
    hq.hqmq_decode_batch(hq.DecodeBatch(params, encs, secs, outs))
    torch.cuda.synchronize()
    for i in range(n):
        assert np.array_equal(outs[i].cpu().numpy().view(np.uint16), singles[i]), i


def test_encode_batch_equals_single_encodes():
    """One launch group for many tensors of a shape must give each tensor exactly hqmq_encode's bytes
    (40 tensors: two groups; the second re-uses the workspace slices of the first)."""
    B, H, T, S = 2, 2, 131, 16
    n = 40
    cb = hq.hqmq_build_codebooks(4, n, H, S)
    xs, secs, singles = [], [], []
    for i in range(n):
        x = _lognormal_tensor(B, H, T, seed=300 + i, sigma_g=0.4 + 0.02 * i).to(DEV)
        sec = cb[i, i % 2].contiguous().to(DEV)
        xs.append(x)
        secs.append(sec)
        singles.append(gpu_encode(x, sec))
    params = hq.params_for(xs[0], S)
    encs = [hq.alloc_encoded(params, DEV) for _ in range(n)]
    for e in encs:
        e.codes.fill_(-1)
    ws = hq.alloc_batch_workspace(params, n, DEV)
    ws.fill_(0xAB)
    hq.hqmq_encode_batch(hq.EncodeBatch(params, xs, secs, encs, ws))
    torch.cuda.synchronize()
    for i in range(n):
        g = singles[i]
        total = int(g.n_out[-1])
        assert total > 0
        assert torch.equal(encs[i].codes, g.bufs.codes), i
        assert torch.equal(encs[i].sigma.view(torch.int16), g.bufs.sigma.view(torch.int16)), i
        assert torch.equal(encs[i].flags, g.bufs.flags) and torch.equal(encs[i].row_off, g.bufs.row_off), i
        assert torch.equal(encs[i].n_outliers, g.bufs.n_outliers) and int(encs[i].status[0]) == 0, i
        assert torch.equal(encs[i].outliers[:total].view(torch.int16), g.bufs.outliers[:total].view(torch.int16)), i


def test_thresholds_are_exported_and_can_be_supplied():
    """hqmq_thresholds returns fl(fl(C C) median) per head, bit for bit; feeding those thresholds to
    hqmq_encode_given_thresholds reproduces the plain encode's bytes."""
    B, H, T, S = 2, 4, 257, 16
    x = _lognormal_tensor(B, H, T, seed=41, sigma_g=0.8)
    sec_t, sec = _sec(2, H, S)
    e = oracle.encode(_bits(x), sec)
    x_dev, sec_dev = x.to(DEV), sec_t.to(DEV)
    params = hq.params_for(x_dev, S)
    bufs = hq.alloc_encoded(params, DEV)
    ws = hq.alloc_workspace(params, DEV)
    hq.hqmq_encode(params, x_dev, sec_dev, bufs, ws)
    thr = hq.hqmq_thresholds(params, ws)
    torch.cuda.synchronize()
    c = float(np.float32(3.0))
    want = (c * c) * e.m2
    assert np.array_equal(thr.cpu().numpy().view(np.uint64), want.view(np.uint64))
    again = hq.alloc_encoded(params, DEV)
    ws.fill_(0x5A)
    hq.hqmq_encode_given_thresholds(params, x_dev, sec_dev, thr, again, ws)
    torch.cuda.synchronize()
    total = int(bufs.n_outliers[-1])
    assert total == int(e.n_out[-1]) > 0
    for a, b in ((again.codes, bufs.codes), (again.flags, bufs.flags), (again.row_off, bufs.row_off),
                 (again.n_outliers, bufs.n_outliers), (again.sigma.view(torch.int16), bufs.sigma.view(torch.int16)),
                 (again.outliers[:total].view(torch.int16), bufs.outliers[:total].view(torch.int16))):
        assert torch.equal(a, b)


@pytest.mark.parametrize("T_new", [1, 3])
def test_incremental_encode_of_appended_tokens(T_new):
    """The generation-step setting: a few new token rows per sequence, encoded against thresholds
    frozen from the prefill (here: of a 300-token tensor of the same law).  Parity with the oracle run
    on the same rows with the same thresholds; the decode round trip on those bytes."""
    B, H, S, b_r = 2, 4, 16, 6
    big = _lognormal_tensor(B, H, 300, seed=51, sigma_g=0.9)
    sec_t, sec = _sec(3, H, S)
    sec_dev = sec_t.to(DEV)
    pb = hq.params_for(big.to(DEV), S, b_r)
    wsb = hq.alloc_workspace(pb, DEV)
    hq.hqmq_encode(pb, big.to(DEV), sec_dev, hq.alloc_encoded(pb, DEV), wsb)
    thr = hq.hqmq_thresholds(pb, wsb)
    torch.cuda.synchronize()

    new = _lognormal_tensor(B, H, 40, seed=52, sigma_g=0.9)[:, :, :T_new].contiguous() * 1.5   # a few spill over
    new = new.to(torch.float16)
    xb = _bits(new)
    e = oracle.encode(xb, sec, b_r=b_r, thresholds=thr.cpu().numpy())
    x_dev = new.to(DEV)
    params = hq.params_for(x_dev, S, b_r)
    n_chunks = B * H * T_new * 32
    bufs = hq.alloc_encoded(params, DEV, outlier_capacity=n_chunks)      # any chunk may be flagged here
    ws = hq.alloc_workspace(params, DEV)
    ws.fill_(0xAB)
    hq.hqmq_encode_given_thresholds(params, x_dev, sec_dev, thr, bufs, ws)
    torch.cuda.synchronize()
    n_out = bufs.n_outliers.cpu().numpy().view(np.uint32)
    total = int(n_out[-1])
    from gpu_util import GpuEncoded
    g = GpuEncoded(params, bufs, bufs.codes.cpu().numpy().view(np.uint32), bufs.sigma.cpu().numpy().view(np.uint16),
                   bufs.flags.cpu().numpy().view(np.uint32), bufs.row_off.cpu().numpy().view(np.uint32), n_out,
                   bufs.outliers[:total].cpu().numpy().view(np.uint16).reshape(total, 4),
                   int(bufs.status.cpu().numpy().view(np.uint32)[0]))
    stats = compare_encode(g, e, xb, sec)
    want, r_hat = oracle.decode(g.codes, g.sigma, g.flags, g.row_off, g.outliers, sec, B, H, T_new, b_r, True)
    got = gpu_decode(params, bufs, sec_dev, x_dev)
    stats["decode_rel_err"] = compare_decode(got, want, r_hat, e.flag)
    print(stats, flush=True)
    assert 0 < stats["outliers"] < n_chunks


@pytest.mark.parametrize("D,B,H,T,S,b_r", [
    (128, 1, 8, 1, 256, 6),     # one appended token of the headline shape: one row per workgroup, all waves on one pass
    (128, 3, 2, 2, 512, 8),     # two rows per workgroup; 8-wave workgroups (S = 512)
    (128, 1, 2, 1, 1, 3),       # fewer groups of secondaries than waves
    (128, 2, 3, 1, 40, 4),      # 3 groups over 4 waves
    (128, 1, 2, 65, 96, 4),     # a full workgroup and one of a single row
    (128, 2, 2, 66, 24, 6),     # ... and one of two rows
    (128, 1, 3, 130, 16, 6),    # three workgroups per segment, the last with two rows
    (128, 4, 8, 128, 64, 6),    # 4096 rows, 64 workgroups: the largest tensor the short form takes
    (128, 8, 8, 1, 256, 6),     # a generation step of 8 sequences: one workgroup per head takes all batch entries
    (128, 4, 2, 2, 64, 6),      # ... 8 rows per head: one pass of the four waves exactly
    (128, 3, 3, 3, 24, 4),      # 9 rows per head: back to one workgroup per (batch entry, head)
    (128, 5, 2, 3, 512, 6),     # 15 rows per head on 8-wave workgroups
    (128, 2, 2, 1, 16, 6),      # two batch entries of one row: one cooperative pass for both
    (96, 2, 4, 1, 192, 4),      # other head dimensions: the flat kernel's short form
    (64, 1, 8, 3, 192, 4),
    (45, 2, 2, 5, 48, 4),
])
def test_short_tensors_with_known_thresholds(D, B, H, T, S, b_r):
    """Tensors of a few rows whose thresholds are known beforehand (supplied, or extraction off) take the
    two-launch form of the encode: parity with the oracle in both modes, and bytes equal to those of the
    same rows encoded as part of a tensor long enough to take the general form (thresholds supplied)."""
    print(f"case D={D} B={B} H={H} T={T} S={S} b_r={b_r}", flush=True)
    x = _lognormal_tensor(B, H, T, seed=7 * T + S + D, sigma_g=1.0, D=D)
    sec_t, sec = _sec(S % 17, H, S)
    sec_dev, x_dev, xb = sec_t.to(DEV), x.to(DEV), _bits(x)
    nc = -(-D // 4)
    # extraction off
    stats, e0, g0 = _roundtrip(x, S, b_r, seed=S % 17, flags=hq.HQMQ_FLAG_NO_OUTLIERS | hq.HQMQ_FLAG_CHECK_FINITE)
    assert g0.status == 0
    # supplied thresholds that flag a fair share of the chunks
    r2 = e0.r2
    thr_np = np.array([np.quantile(r2.reshape(B, H, T * nc)[:, h], 0.8) for h in range(H)])
    thr = torch.from_numpy(thr_np).to(DEV)
    e = oracle.encode(xb, sec, b_r=b_r, thresholds=thr_np)
    params = hq.params_for(x_dev, S, b_r)
    bufs = hq.alloc_encoded(params, DEV, outlier_capacity=B * H * T * nc)
    ws = hq.alloc_workspace(params, DEV)
    ws.fill_(0x5A)
    for t in (bufs.codes, bufs.flags, bufs.row_off, bufs.n_outliers, bufs.status):
        t.fill_(-1)
    hq.hqmq_encode_given_thresholds(params, x_dev, sec_dev, thr, bufs, ws)
    torch.cuda.synchronize()
    assert torch.equal(hq.hqmq_thresholds(params, ws), thr)
    from gpu_util import GpuEncoded
    total = int(bufs.n_outliers[-1])
    g = GpuEncoded(params, bufs, bufs.codes.cpu().numpy().view(np.uint32), bufs.sigma.cpu().numpy().view(np.uint16),
                   bufs.flags.cpu().numpy().view(np.uint32), bufs.row_off.cpu().numpy().view(np.uint32),
                   bufs.n_outliers.cpu().numpy().view(np.uint32),
                   bufs.outliers[:total].cpu().numpy().view(np.uint16).reshape(total, 4), int(bufs.status.item()))
    stats = compare_encode(g, e, xb, sec)
    assert stats["outliers"] > 0 or T * nc < 8
    # the same rows at the front of a long tensor (general form: separate operand table, scan and gather
    # kernels): code words, scales and flag words of those rows must be the same bytes
    T_long = 5000 if B * H * 5000 > 4096 else 9000
    long = torch.zeros(B, H, T_long, D, dtype=torch.float16)
    long[:, :, :T] = x
    pl = hq.params_for(long.to(DEV), S, b_r)
    bl = hq.alloc_encoded(pl, DEV, outlier_capacity=B * H * T_long * nc)
    hq.hqmq_encode_given_thresholds(pl, long.to(DEV), sec_dev, thr, bl, hq.alloc_workspace(pl, DEV))
    torch.cuda.synchronize()
    rows_long = (torch.arange(B * H).view(-1, 1) * T_long + torch.arange(T).view(1, -1)).reshape(-1).to(DEV)
    assert torch.equal(bl.codes[rows_long], bufs.codes)
    assert torch.equal(bl.flags[rows_long], bufs.flags)
    assert torch.equal(bl.sigma[rows_long].view(torch.int16), bufs.sigma.view(torch.int16))


def test_batched_incremental_encode_equals_single_calls():
    B, H, S, T_new, n = 2, 4, 16, 2, 5
    cb = hq.hqmq_build_codebooks(6, n, H, S)
    xs, secs, thrs, singles = [], [], [], []
    for i in range(n):
        x = (_lognormal_tensor(B, H, 8, seed=400 + i, sigma_g=0.8)[:, :, :T_new].contiguous()).to(DEV)
        sec = cb[i, 0].contiguous().to(DEV)
        thr = torch.full((H,), 4.0 + i, dtype=torch.float64, device=DEV)
        params = hq.params_for(x, S)
        bufs = hq.alloc_encoded(params, DEV, outlier_capacity=B * H * T_new * 32)
        hq.hqmq_encode_given_thresholds(params, x, sec, thr, bufs, hq.alloc_workspace(params, DEV))
        xs.append(x), secs.append(sec), thrs.append(thr), singles.append(bufs)
    encs = [hq.alloc_encoded(params, DEV, outlier_capacity=B * H * T_new * 32) for _ in range(n)]
    batch = hq.EncodeBatch(params, xs, secs, encs, hq.alloc_batch_workspace(params, n, DEV))
    hq.hqmq_encode_batch_given_thresholds(batch, thrs)
    torch.cuda.synchronize()
    for a, b in zip(encs, singles):
        total = int(b.n_outliers[-1])
        assert total > 0
        assert torch.equal(a.codes, b.codes) and torch.equal(a.flags, b.flags) and torch.equal(a.row_off, b.row_off)
        assert torch.equal(a.n_outliers, b.n_outliers)
        assert torch.equal(a.sigma.view(torch.int16), b.sigma.view(torch.int16))
        assert torch.equal(a.outliers[:total].view(torch.int16), b.outliers[:total].view(torch.int16))


@pytest.mark.parametrize("D", [128, 96])
def test_check_finite_flag_reports_infinities_and_nans(D):
    """The paper does not define the encode of a non-finite value; the library's contract is a status bit
    when HQMQ_FLAG_CHECK_FINITE is set, in every mode of the encode (own median, extraction off, supplied
    thresholds), and code words that stay inside the codebook so that a decode of the result is safe."""
    B, H, T, S = 1, 3, 700, 48
    clean = _lognormal_tensor(B, H, T, seed=31, D=D)
    sec_t, sec = _sec(2, H, S)
    sec_dev = sec_t.to(DEV)
    CF, NF = hq.HQMQ_FLAG_CHECK_FINITE, hq.HQMQ_STATUS_NONFINITE
    # finite input: the flag changes nothing, and the result is the oracle's
    stats, e, g = _roundtrip(clean, S, seed=2, flags=CF)
    plain = gpu_encode(clean.to(DEV), sec_dev, flags=0)
    assert g.status == 0 and plain.status == 0
    for f in ("codes", "sigma", "flags", "row_off", "n_out", "outliers"):
        assert np.array_equal(getattr(g, f), getattr(plain, f)), f
    nc = -(-D // 4)
    for what in ("inf", "nan", "both"):
        x = clean.clone()
        if what in ("inf", "both"):
            x[0, 1, 333, 5] = float("-inf")
        if what in ("nan", "both"):
            x[0, 2, 699, D - 1] = float("nan")
        xd = x.to(DEV)
        for flags in (CF, CF | hq.HQMQ_FLAG_NO_OUTLIERS):
            g = gpu_encode(xd, sec_dev, flags=flags)
            assert g.status & NF, (what, flags)
            k, _ = oracle.unpack_rows(g.codes, S, 6, nc)
            assert (k < 24 * S).all()
            gpu_decode(g.params, g.bufs, sec_dev, xd)          # stays in bounds, whatever it returns
        for flags in (0, hq.HQMQ_FLAG_NO_OUTLIERS):
            assert not (gpu_encode(xd, sec_dev, flags=flags).status & NF)   # only reported on request
        # supplied thresholds
        params = hq.params_for(xd, S, 6, 3.0, CF)
        bufs = hq.alloc_encoded(params, DEV, B * H * T * nc)
        thr = torch.full((H,), 50.0, dtype=torch.float64, device=DEV)
        hq.hqmq_encode_given_thresholds(params, xd, sec_dev, thr, bufs, hq.alloc_workspace(params, DEV))
        torch.cuda.synchronize()
        assert int(bufs.status.item()) & NF


def test_concurrent_encodes_from_two_threads():
    """Calls on distinct buffers and streams may come from different host threads: every thread's results
    equal those of the same calls made one after the other."""
    import threading
    S = 64
    xs = [_lognormal_tensor(1, 4, 900 + 50 * i, seed=40 + i).to(DEV) for i in range(2)]
    sec_dev = _sec(3, 4, S)[0].to(DEV)
    want = [gpu_encode(x, sec_dev) for x in xs]
    got = [None, None]
    errors = []

    def worker(i):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                params = hq.params_for(xs[i], S)
                ws = hq.alloc_workspace(params, DEV)
                for _ in range(20):
                    bufs = hq.alloc_encoded(params, DEV)
                    hq.hqmq_encode(params, xs[i], sec_dev, bufs, ws, stream=stream)
                    out = torch.empty_like(xs[i])
                    hq.hqmq_decode(params, bufs, sec_dev, out, stream=stream)
                stream.synchronize()
                got[i] = (bufs, out)
        except Exception as exc:       # noqa: BLE001 - reported by the main thread
            errors.append(exc)
    torch.cuda.synchronize()
    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for i in range(2):
        bufs, out = got[i]
        assert np.array_equal(bufs.codes.cpu().numpy().view(np.uint32), want[i].codes)
        assert np.array_equal(bufs.flags.cpu().numpy().view(np.uint32), want[i].flags)
        assert np.array_equal(bufs.row_off.cpu().numpy().view(np.uint32), want[i].row_off)
        assert np.array_equal(bufs.sigma.cpu().numpy().view(np.uint16), want[i].sigma)
        ref = gpu_decode(want[i].params, want[i].bufs, sec_dev, xs[i])
        assert np.array_equal(out.cpu().numpy().view(np.uint16), ref)


def _sweep_cases(n, seed):
    """Seeded random encode / decode cases over head dimensions, codebook sizes, radius widths, shapes (ragged
    tails, workgroup and tile edges), multipliers and flags, a quarter of them with the chunk norms packed into
    a narrow band (the median select's overflow paths); sized so that the oracle takes about a second each."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        D = int(rng.choice([128, 128, 96, 64, int(rng.integers(1, 129))]))
        S = int(rng.choice([1, 2, 3, 5, 16, 24, 48, 64, 96, 100, 192, 255, 256, 257, 384, 512]))
        b_r = int(rng.integers(1, 9))
        B, H = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        nc = -(-D // 4)
        budget = 1.5e7
        max_t = max(1, int(budget / (B * H * nc * 24 * S)))
        T = int(rng.integers(1, min(max_t, 5000) + 1))
        if rng.random() < 0.2:
            T = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 2047, 2048, 2049]))
            if B * H * T * nc * 24 * S > 4 * budget:
                continue
        C = float(rng.choice([3.0, 3.0, 1.5, 10.0, 0.7]))
        flags = int(rng.choice([0, 0, 0, 0, 0, 0, 0, 1, 2, 3]))
        sg = float(rng.choice([0.3, 0.7, 1.2]))
        spread = float(rng.choice([0.001, 0.004, 0.03, 0.2])) if rng.random() < 0.25 else 0.0
        cases.append((D, S, b_r, B, H, T, C, flags, sg, spread, int(rng.integers(1, 10 ** 6))))
    return cases


@pytest.mark.parametrize("D,S,b_r,B,H,T,C,flags,sg,spread,seed", _sweep_cases(40, seed=20261128))
def test_randomized_sweep(D, S, b_r, B, H, T, C, flags, sg, spread, seed):
    print(f"case D={D} S={S} b_r={b_r} B={B} H={H} T={T} C={C} flags={flags} sg={sg} spread={spread} seed={seed}",
          flush=True)
    x = _lognormal_tensor(B, H, T, seed=seed, sigma_g=sg, D=D)
    if spread:
        gen = torch.Generator().manual_seed(seed + 1)
        mag = (1.0 + spread * (2.0 * torch.rand(x.shape, generator=gen) - 1.0)) * [1e-3, 1.0, 50.0][seed % 3]
        x = (mag * torch.where(torch.rand(x.shape, generator=gen) < 0.5, -1.0, 1.0)).half()
        x[..., ::5, :4] *= 5.0
    _roundtrip(x, S, b_r=b_r, Cmul=C, seed=seed % 100, flags=flags)


def test_deterministic_bytes():
    x = _lognormal_tensor(1, 4, 300, seed=15).to(DEV)
    sec_t, _ = _sec(0, 4, 64)
    a = gpu_encode(x, sec_t.to(DEV))
    b = gpu_encode(x, sec_t.to(DEV))
    for f in ("codes", "sigma", "flags", "row_off", "n_out", "outliers"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f


def test_codebooks_of_library_and_oracle_agree():
    for seed in (0, 1, 7, 42, 1337):
        lib = hq.hqmq_build_codebooks(seed, 2, 4, 64).numpy()
        ora = oracle.build_codebooks(seed, 2, 4, 64)
        ulp = np.abs(lib.view(np.int32).astype(np.int64) - ora.view(np.int32).astype(np.int64))
        assert ulp.max() <= 2
