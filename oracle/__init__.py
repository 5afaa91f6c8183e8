"""HQMQ reference oracle: Python face of ``hqmq_oracle.c``.

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the bench's CPU-baseline
leg may import this package; the GPU library never does, and this package never imports
the GPU library.  All arithmetic lives in the C file (plain fp64, written from the paper);
this module marshals numpy arrays, strings the steps together in the order of Alg. 1, and
holds the closed-form bit accounting of Sec. 3 / Eq. (2).
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hqmq_oracle.c")
_LIB = os.path.join(_HERE, "libhqmq_oracle.so")

NC = 32  # most chunks a packed row may have (head dimension 128)


def chunks_per_row(D: int) -> int:
    """Quaternion chunks of a head vector of D elements: ceil(D / 4); a head dimension that is not
    a multiple of 4 is zero-padded to the next one (App. "Padding wrapper for d_h not divisible by 4")."""
    nc = (int(D) + 3) // 4
    if not 1 <= nc <= NC:
        raise ValueError("the oracle packs rows of 1..128 elements")
    return nc


def row_words(D: int, w: int) -> int:
    """32-bit words of one packed row: ceil(chunks * w / 32)."""
    return (chunks_per_row(D) * w + 31) // 32


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every rounding where the
    source puts it; OpenMP only drives the parallel-for over rows of the search."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fopenmp",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _declare(_lib)
    return _lib


_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
_u16p = np.ctypeslib.ndpointer(np.uint16, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")


def _declare(L):
    L.hqo_half_to_double.restype = C.c_double
    L.hqo_half_to_double.argtypes = [C.c_uint16]
    L.hqo_double_to_half.restype = C.c_uint16
    L.hqo_double_to_half.argtypes = [C.c_double]
    L.hqo_hamilton.restype = None
    L.hqo_hamilton.argtypes = [_f64p, _f64p, _f64p]
    L.hqo_primary.restype = None
    L.hqo_primary.argtypes = [C.c_int, _f64p]
    L.hqo_codeword.restype = None
    L.hqo_codeword.argtypes = [_f32p, C.c_int, C.c_int, _f64p]
    L.hqo_build_codebooks.restype = None
    L.hqo_build_codebooks.argtypes = [C.c_uint64, C.c_int, C.c_int, C.c_int, _f32p]
    L.hqo_norm2.restype = None
    L.hqo_norm2.argtypes = [_u16p, C.c_int64, _f64p]
    L.hqo_lower_median.restype = C.c_double
    L.hqo_lower_median.argtypes = [_f64p, C.c_int64]
    L.hqo_head_medians.restype = None
    L.hqo_head_medians.argtypes = [_f64p, C.c_int, C.c_int, C.c_int, C.c_int, _f64p]
    L.hqo_flags.restype = None
    L.hqo_flags.argtypes = [_f64p, _f64p, C.c_float, C.c_int, C.c_int, C.c_int, C.c_int,
                            C.c_int, _u8p]
    L.hqo_extract_outliers.restype = C.c_int64
    L.hqo_extract_outliers.argtypes = [_u16p, _u8p, C.c_int, C.c_int, C.c_int, C.c_int, _u32p, _u32p,
                                       _u32p, _u16p, C.c_int64]
    L.hqo_row_sigma.restype = None
    L.hqo_row_sigma.argtypes = [_f64p, _u8p, C.c_int64, C.c_int, _u16p]
    L.hqo_score.restype = C.c_double
    L.hqo_score.argtypes = [_u16p, _f32p, C.c_int, C.c_int]
    L.hqo_search_chunk.restype = None
    L.hqo_search_chunk.argtypes = [_u16p, _f32p, C.c_int, C.POINTER(C.c_int32),
                                   C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.hqo_radius_code.restype = C.c_int32
    L.hqo_radius_code.argtypes = [C.c_double, C.c_uint16, C.c_int]
    L.hqo_index_bits.restype = C.c_int
    L.hqo_index_bits.argtypes = [C.c_int]
    L.hqo_search_rows.restype = None
    L.hqo_search_rows.argtypes = [_u16p, _u8p, _u16p, _f32p, C.c_int, C.c_int, C.c_int, C.c_int,
                                  C.c_int, C.c_int, C.c_void_p, _i32p, _f64p, _f64p, _i32p]
    L.hqo_pack_row.restype = None
    L.hqo_pack_row.argtypes = [_u32p, C.c_int, C.c_int, _u32p]
    L.hqo_unpack_row.restype = None
    L.hqo_unpack_row.argtypes = [_u32p, C.c_int, C.c_int, _u32p]
    L.hqo_pack_rows.restype = None
    L.hqo_pack_rows.argtypes = [_i32p, _i32p, _u8p, C.c_int64, C.c_int, C.c_int, C.c_int, _u32p]
    L.hqo_decode64.restype = None
    L.hqo_decode64.argtypes = [_u32p, _u16p, _u32p, _u32p, _u16p, _f32p, C.c_int, C.c_int,
                               C.c_int, C.c_int, C.c_int, C.c_int, _u16p, C.c_void_p, _f64p]
    L.hqo_attend.restype = None
    L.hqo_attend.argtypes = [_u16p, _f64p, _f64p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                             C.c_double, _u16p, _f64p]
    L.hqo_attend_lse.restype = None
    L.hqo_attend_lse.argtypes = [_u16p, _f64p, _f64p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                 C.c_double, _u16p, _f64p, _f64p]
    L.hqo_attend_masked.restype = None
    L.hqo_attend_masked.argtypes = [_u16p, _f64p, _f64p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                    C.c_double, C.c_void_p, _u16p, _f64p, _f64p]
    L.hqo_decode.restype = None
    L.hqo_decode.argtypes = [_u32p, _u16p, _u32p, _u32p, _u16p, _f32p, C.c_int, C.c_int,
                             C.c_int, C.c_int, C.c_int, C.c_int, _u16p, C.c_void_p]


# --------------------------------------------------------------------------------------
# thin wrappers of the single steps
# --------------------------------------------------------------------------------------

def set_threads(n: int) -> None:
    """Number of threads of the row-parallel search (0/None: OpenMP default)."""
    omp = C.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(n))


def max_threads() -> int:
    omp = C.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


def set_threads(n: int) -> None:
    """Number of host threads the oracle's parallel-for over rows uses from now on."""
    omp = C.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(n))


def primary(p: int) -> np.ndarray:
    q = np.zeros(4)
    lib().hqo_primary(int(p), q)
    return q


def primaries() -> np.ndarray:
    return np.stack([primary(p) for p in range(24)])


def hamilton(a, b) -> np.ndarray:
    out = np.zeros(4)
    lib().hqo_hamilton(np.ascontiguousarray(a, np.float64), np.ascontiguousarray(b, np.float64), out)
    return out


def codeword(sec_head: np.ndarray, k: int) -> np.ndarray:
    sec_head = np.ascontiguousarray(sec_head, np.float32)
    out = np.zeros(4)
    lib().hqo_codeword(sec_head, sec_head.shape[0], int(k), out)
    return out


def joint_codebook(sec_head: np.ndarray) -> np.ndarray:
    S = sec_head.shape[0]
    return np.stack([codeword(sec_head, k) for k in range(24 * S)])


def build_codebooks(seed: int, n_layers: int, n_heads: int, S: int) -> np.ndarray:
    out = np.zeros((n_layers, 2, n_heads, S, 4), np.float32)
    lib().hqo_build_codebooks(int(seed), n_layers, n_heads, S, out.reshape(-1))
    return out


def half_to_double(bits) -> np.ndarray:
    bits = np.asarray(bits, np.uint16)
    f = lib().hqo_half_to_double
    return np.array([f(int(b)) for b in bits.reshape(-1)]).reshape(bits.shape)


def double_to_half(v) -> np.ndarray:
    v = np.asarray(v, np.float64)
    f = lib().hqo_double_to_half
    return np.array([f(float(a)) for a in v.reshape(-1)], np.uint16).reshape(v.shape)


def norm2(x_bits: np.ndarray) -> np.ndarray:
    x_bits = np.ascontiguousarray(x_bits, np.uint16)
    n = x_bits.size // 4
    r2 = np.zeros(n)
    lib().hqo_norm2(x_bits.reshape(-1), n, r2)
    return r2.reshape(x_bits.shape[:-1] + (x_bits.shape[-1] // 4,))


def lower_median(v) -> float:
    v = np.ascontiguousarray(v, np.float64).reshape(-1)
    return float(lib().hqo_lower_median(v, v.size))


def index_bits(S: int) -> int:
    return int(lib().hqo_index_bits(int(S)))


def search_chunk(x4_bits, sec_head):
    x4_bits = np.ascontiguousarray(x4_bits, np.uint16)
    sec_head = np.ascontiguousarray(sec_head, np.float32)
    k, b, s = C.c_int32(), C.c_double(), C.c_double()
    lib().hqo_search_chunk(x4_bits, sec_head, sec_head.shape[0], C.byref(k), C.byref(b), C.byref(s))
    return k.value, b.value, s.value


def score(x4_bits, sec_head, k: int) -> float:
    x4_bits = np.ascontiguousarray(x4_bits, np.uint16)
    sec_head = np.ascontiguousarray(sec_head, np.float32)
    return float(lib().hqo_score(x4_bits, sec_head, sec_head.shape[0], int(k)))


def radius_code(r2: float, sigma16: int, b_r: int) -> int:
    return int(lib().hqo_radius_code(float(r2), int(sigma16), int(b_r)))


def pack_row(code32, w: int) -> np.ndarray:
    """Pack the codes of one row (as many chunks as code32 has entries, at most 32)."""
    code32 = np.ascontiguousarray(code32, np.uint32)
    nc = code32.size
    words = np.zeros((nc * w + 31) // 32, np.uint32)
    lib().hqo_pack_row(code32, nc, w, words)
    return words


def unpack_row(words, w: int, nc: int = NC) -> np.ndarray:
    words = np.ascontiguousarray(words, np.uint32)
    code32 = np.zeros(nc, np.uint32)
    lib().hqo_unpack_row(words, nc, w, code32)
    return code32


def unpack_rows(codes: np.ndarray, S: int, b_r: int, nc: int = NC):
    """codes [rows][row_words] -> (k [rows][nc], r_q [rows][nc]) with the oracle's bit layout."""
    w_idx = index_bits(S)
    w = w_idx + b_r
    codes = np.ascontiguousarray(codes, np.uint32).reshape(-1, (nc * w + 31) // 32)
    k = np.zeros((codes.shape[0], nc), np.int64)
    rq = np.zeros((codes.shape[0], nc), np.int64)
    for i in range(codes.shape[0]):
        c = unpack_row(codes[i], w, nc).astype(np.int64)
        k[i] = c & ((1 << w_idx) - 1)
        rq[i] = c >> w_idx
    return k, rq


# --------------------------------------------------------------------------------------
# the whole path, steps in the order of Alg. 1
# --------------------------------------------------------------------------------------

@dataclass
class Encoded:
    """Everything the encode of one (layer, role) tensor produces, plus diagnostics."""
    B: int
    H: int
    T: int
    D: int
    S: int
    b_r: int
    r2: np.ndarray          # [rows, Nc] fp64 squared norms (Nc = ceil(D / 4) chunks per row)
    m2: np.ndarray          # [H] lower median of r2 per head
    flag: np.ndarray        # [rows, Nc] uint8
    flags: np.ndarray       # [rows] uint32 flag words
    row_off: np.ndarray     # [rows + 1] uint32
    n_out: np.ndarray       # [H + 1] uint32
    outliers: np.ndarray    # [n_out[H], 4] uint16 (fp16 bit patterns)
    sigma: np.ndarray       # [rows] uint16 (fp16 bit patterns)
    k: np.ndarray           # [rows, Nc] int32, -1 where flagged / not searched
    rq: np.ndarray          # [rows, Nc] int32, -1 where flagged / not searched
    best: np.ndarray        # [rows, Nc] fp64 best score
    second: np.ndarray      # [rows, Nc] fp64 runner-up score
    codes: np.ndarray       # [rows, ceil(Nc w / 32)] uint32
    searched: np.ndarray    # [rows] bool


def encode(x_bits: np.ndarray, sec: np.ndarray, b_r: int = 6, Cmul: float = 3.0,
           use_outliers: bool = True, rows=None, thresholds=None) -> Encoded:
    """Encode one fp16 tensor [B, H, T, D] (uint16 bit patterns), D <= 128, against the secondary
    codebooks sec [H, S, 4] (fp32) of its (layer, role).  A D that is not a multiple of 4 is
    zero-padded to the next one first (App. "Padding wrapper for d_h not divisible by 4").  `rows`: optional boolean mask or
    index list of the rows whose (expensive) search is run; the O(n) steps always cover the
    whole tensor.  `thresholds`: fp64 [H] on squared norms, supplied instead of the batch's
    own C^2 * median (the incremental setting: a chunk is flagged iff r^2 > thresholds[h])."""
    L = lib()
    x_bits = np.ascontiguousarray(x_bits, np.uint16)
    B, H, T, D = x_bits.shape
    nc = chunks_per_row(D)
    if D != 4 * nc:
        padded = np.zeros((B, H, T, 4 * nc), np.uint16)  # +0.0 in the missing elements
        padded[..., :D] = x_bits
        x_bits = padded
    sec = np.ascontiguousarray(sec, np.float32)
    assert sec.shape[0] == H and sec.shape[2] == 4
    S = sec.shape[1]
    n_rows = B * H * T
    n_chunks = n_rows * nc
    flat = x_bits.reshape(-1)

    r2 = np.zeros(n_chunks)
    L.hqo_norm2(flat, n_chunks, r2)
    m2 = np.zeros(H)
    L.hqo_head_medians(r2, B, H, T, nc, m2)
    flag = np.zeros(n_chunks, np.uint8)
    if thresholds is None:
        L.hqo_flags(r2, m2, float(Cmul), int(bool(use_outliers)), B, H, T, nc, flag)
    else:
        # the flag rule compares against fl(fl(C C) m): with C = 1 that is m itself
        L.hqo_flags(r2, np.ascontiguousarray(thresholds, np.float64), 1.0, 1, B, H, T, nc, flag)

    flags = np.zeros(n_rows, np.uint32)
    row_off = np.zeros(n_rows + 1, np.uint32)
    n_out = np.zeros(H + 1, np.uint32)
    cap = int(flag.sum())
    payload = np.zeros((max(cap, 1), 4), np.uint16)
    total = L.hqo_extract_outliers(flat, flag, B, H, T, nc, flags, row_off, n_out,
                                   payload.reshape(-1), cap)
    assert total == cap
    payload = payload[:cap]

    sigma = np.zeros(n_rows, np.uint16)
    L.hqo_row_sigma(r2, flag, n_rows, nc, sigma)

    if rows is None:
        sel = None
        searched = np.ones(n_rows, bool)
    else:
        rows = np.asarray(rows)
        if rows.dtype == bool:
            searched = rows.copy()
        else:
            searched = np.zeros(n_rows, bool)
            searched[rows] = True
        sel = np.ascontiguousarray(searched.astype(np.uint8))
    k = np.zeros(n_chunks, np.int32)
    rq = np.zeros(n_chunks, np.int32)
    best = np.zeros(n_chunks)
    second = np.zeros(n_chunks)
    L.hqo_search_rows(flat, flag, sigma, sec.reshape(-1), B, H, T, nc, S, b_r,
                      None if sel is None else sel.ctypes.data, k, best, second, rq)

    w = index_bits(S) + b_r
    codes = np.zeros((n_rows, (nc * w + 31) // 32), np.uint32)
    L.hqo_pack_rows(k, rq, flag, n_rows, nc, S, b_r, codes.reshape(-1))

    return Encoded(B, H, T, D, S, b_r, r2.reshape(n_rows, nc), m2, flag.reshape(n_rows, nc),
                   flags, row_off, n_out, payload, sigma, k.reshape(n_rows, nc),
                   rq.reshape(n_rows, nc), best.reshape(n_rows, nc),
                   second.reshape(n_rows, nc), codes, searched)


def decode(codes, sigma, flags, row_off, outliers, sec, B, H, T, b_r, want_r_hat=False, D=4 * NC):
    """Decode to fp16 bit patterns [B, H, T, D] (the padding elements of a D that is not a multiple
    of 4 are cut off again); optionally also r_hat [rows, ceil(D / 4)]."""
    sec = np.ascontiguousarray(sec, np.float32)
    S = sec.shape[1]
    n_rows = B * H * T
    nc = chunks_per_row(D)
    out = np.zeros(n_rows * nc * 4, np.uint16)
    r_hat = np.zeros(n_rows * nc) if want_r_hat else None
    outliers = np.ascontiguousarray(outliers, np.uint16).reshape(-1)
    if outliers.size == 0:
        outliers = np.zeros(4, np.uint16)
    lib().hqo_decode(np.ascontiguousarray(codes, np.uint32).reshape(-1),
                     np.ascontiguousarray(sigma, np.uint16),
                     np.ascontiguousarray(flags, np.uint32),
                     np.ascontiguousarray(row_off, np.uint32), outliers, sec.reshape(-1),
                     B, H, T, nc, S, b_r, out, None if r_hat is None else r_hat.ctypes.data)
    out = np.ascontiguousarray(out.reshape(B, H, T, nc * 4)[..., :D])
    if want_r_hat:
        return out, r_hat.reshape(n_rows, nc)
    return out


def decode64(codes, sigma, flags, row_off, outliers, sec, B, H, T, b_r, D=4 * NC) -> np.ndarray:
    """Reconstruction before the final fp16 rounding, fp64 [B, H, T, D] (outliers widened)."""
    sec = np.ascontiguousarray(sec, np.float32)
    S = sec.shape[1]
    n_rows = B * H * T
    nc = chunks_per_row(D)
    out16 = np.zeros(n_rows * nc * 4, np.uint16)
    out64 = np.zeros(n_rows * nc * 4)
    outliers = np.ascontiguousarray(outliers, np.uint16).reshape(-1)
    if outliers.size == 0:
        outliers = np.zeros(4, np.uint16)
    lib().hqo_decode64(np.ascontiguousarray(codes, np.uint32).reshape(-1),
                       np.ascontiguousarray(sigma, np.uint16), np.ascontiguousarray(flags, np.uint32),
                       np.ascontiguousarray(row_off, np.uint32), outliers, sec.reshape(-1),
                       B, H, T, nc, S, b_r, out16, None, out64)
    return np.ascontiguousarray(out64.reshape(B, H, T, nc * 4)[..., :D])


def attend(q_bits: np.ndarray, K64: np.ndarray, V64: np.ndarray, scale: float, want_lse: bool = False,
           visible=None):
    """Single-query attention (one token per sequence) over a reconstructed cache.
    q_bits: fp16 bit patterns [B, Hq, D]; K64, V64: fp64 [B, H, T, D]; returns (fp16 bits, fp64) and,
    with want_lse, the natural log of the softmax denominator, fp64 [B, Hq].  visible: optional int32
    [B, Hq], query head hq sees only the tokens t < visible[b, hq] (causal limit)."""
    q_bits = np.ascontiguousarray(q_bits, np.uint16)
    K64 = np.ascontiguousarray(K64, np.float64)
    V64 = np.ascontiguousarray(V64, np.float64)
    B, Hq, D = q_bits.shape
    _, H, T, _ = K64.shape
    assert Hq % H == 0 and K64.shape == V64.shape and K64.shape[0] == B and K64.shape[3] == D
    out16 = np.zeros((B, Hq, D), np.uint16)
    out64 = np.zeros((B, Hq, D))
    lse = np.zeros((B, Hq))
    vis = None if visible is None else np.ascontiguousarray(visible, np.int32).reshape(B, Hq)
    lib().hqo_attend_masked(q_bits.reshape(-1), K64.reshape(-1), V64.reshape(-1), B, Hq, H, T, D, float(scale),
                            None if vis is None else vis.ctypes.data, out16.reshape(-1), out64.reshape(-1),
                            lse.reshape(-1))
    if want_lse:
        return out16, out64, lse
    return out16, out64


# --------------------------------------------------------------------------------------
# storage accounting (Sec. 3 "Joint codebook ...", Eq. (2), App. "Bit accounting examples")
# --------------------------------------------------------------------------------------

def bits_per_element(S: int, b_r: int, d_h: int = 128, p: float | None = None,
                     stored: bool = False) -> float:
    """b_HQMQ = (log2(24 S) + b_r)/4 + 16/d_h; with an outlier fraction p (Eq. 2):
    (1-p) b_HQMQ + 16 p + 1/4.  stored=True uses the ceil(log2(24 S)) bits actually kept."""
    idx = index_bits(S) if stored else math.log2(24 * S)
    b = (idx + b_r) / 4.0 + 16.0 / d_h
    if p is not None:
        b = (1.0 - p) * b + 16.0 * p + 1.0 / 4.0
    return b


def padding_overhead(d_h: int) -> float:
    """Relative storage overhead of zero-padding a head of d_h elements to whole chunks:
    ceil(d_h / 4) * 4 / d_h - 1 (App. "Padding wrapper for d_h not divisible by 4")."""
    return chunks_per_row(d_h) * 4.0 / d_h - 1.0
