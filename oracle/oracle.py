"""ctypes front end of the float64 CPU oracle (``vecinfer_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg call this; the GPU library never does, and nothing here
imports the GPU package.

Inputs arrive as the same fp16 / fp32 / uint8 arrays the GPU path receives and
are widened to float64 (exactly) before the C code sees them.  Shapes follow
the paper's notation: D = head dim, d = sub-vector dim, M = D / d sub-spaces,
C = 2^b centroids per sub-space (Sec. 2.2), N tokens in the cache.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vecinfer_oracle.c")
_LIB = os.path.join(_HERE, "libvecinfer_oracle.so")
_lib = None


_SAN_LIB = os.path.join(_HERE, "libvecinfer_oracle_san.so")
# VECINFER_ORACLE_SANITIZED=1 (set before the first call): load the AddressSanitizer +
# UndefinedBehaviorSanitizer build instead.  The process must then have been started with the
# sanitizer runtime preloaded (see build_sanitized); the CPU test tier does that in a child process.
_SANITIZED = os.environ.get("VECINFER_ORACLE_SANITIZED") == "1"


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (``-O2``, OpenMP, no fast-math)."""
    if _SANITIZED:
        return build_sanitized(force)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
               "-ffp-contract=off", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def sanitizer_runtime() -> str:
    """Path of gcc's AddressSanitizer runtime, to be preloaded into a process that loads the sanitized build."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()


def build_sanitized(force: bool = False) -> str:
    """The same source with -fsanitize=address,undefined (-O1, frame pointers kept, no OpenMP so that
    every report points into the oracle): out-of-bounds accesses, misaligned or overflowing
    arithmetic and the like abort the process instead of passing silently."""
    if force or not os.path.exists(_SAN_LIB) or os.path.getmtime(_SAN_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off", "-Wall", "-Wextra",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
               "-Wno-unknown-pragmas", "-o", _SAN_LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SAN_LIB


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        dp, u8p, i64p = C.POINTER(C.c_double), C.POINTER(C.c_uint8), C.POINTER(C.c_int64)
        lib.vo_num_threads.restype = C.c_int
        lib.vo_set_num_threads.argtypes = [C.c_int]
        lib.vo_hadamard.argtypes = [C.c_int, dp]
        lib.vo_hadamard.restype = C.c_int
        lib.vo_smoothing_factors.argtypes = [dp, C.c_int64, C.c_int, dp]
        lib.vo_transform_keys.argtypes = [dp, C.c_int64, C.c_int, dp, dp, dp]
        lib.vo_transform_query.argtypes = [dp, C.c_int, dp, dp, dp]
        lib.vo_vq_encode.argtypes = [dp, C.c_int64, C.c_int, C.c_int, C.c_int, dp, u8p, dp]
        lib.vo_vq_dequantize.argtypes = [u8p, C.c_int64, C.c_int, C.c_int, C.c_int, dp, dp]
        lib.vo_merge_splits.argtypes = [dp, dp, C.c_int, C.c_int, dp, dp]
        lib.vo_encode_batch.argtypes = [dp, dp, dp, C.c_int, C.c_int, C.c_int64, C.c_int,
                                        C.c_int, C.c_int, C.c_int, u8p, dp]
        lib.vo_encode_batch.restype = C.c_int
        lib.vo_decode_batch.argtypes = [dp, dp, dp, dp, u8p, u8p, i64p, C.c_int, C.c_int,
                                        C.c_int, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int,
                                        C.c_int, C.c_int64, dp, dp]
        lib.vo_decode_batch.restype = C.c_int
        lib.vo_decode_residual_batch.argtypes = [dp, dp, dp, dp, u8p, u8p, i64p, dp, dp, i64p, C.c_int, C.c_int,
                                                 C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int,
                                                 C.c_int, dp, dp]
        lib.vo_decode_residual_batch.restype = C.c_int
        lib.vo_kmeans_update.argtypes = [dp, u8p, C.c_int64, C.c_int, C.c_int, C.c_int, dp, dp, i64p]
        u16p = C.POINTER(C.c_uint16)
        lib.vo_vq_encode_g.argtypes = [dp, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, dp, u16p, dp]
        lib.vo_vq_dequantize_g.argtypes = [u16p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, dp, dp]
        lib.vo_encode_batch_g.argtypes = [dp, dp, dp, C.c_int, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_int,
                                          C.c_int, C.c_int, u16p, dp]
        lib.vo_encode_batch_g.restype = C.c_int
        lib.vo_decode_batch_g.argtypes = [dp, dp, dp, dp, u16p, u16p, i64p, C.c_int, C.c_int, C.c_int, C.c_int64,
                                          C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, dp, dp]
        lib.vo_decode_batch_g.restype = C.c_int
        lib.vo_decode_residual_batch_g.argtypes = [dp, dp, dp, dp, u16p, u16p, i64p, dp, dp, i64p, C.c_int, C.c_int,
                                                   C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int,
                                                   C.c_int, C.c_int, C.c_int, dp, dp]
        lib.vo_decode_residual_batch_g.restype = C.c_int
        lib.vo_kmeans_update_g.argtypes = [dp, u16p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, dp, dp, i64p]
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _u8p(a):
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


def _u16p(a):
    return a.ctypes.data_as(C.POINTER(C.c_uint16))


def num_threads() -> int:
    return int(_load().vo_num_threads())


def set_num_threads(n: int) -> None:
    _load().vo_set_num_threads(int(n))


def hadamard(D: int) -> np.ndarray:
    """Orthonormal Walsh-Hadamard matrix H_D of Eq. 5 (Sylvester order)."""
    H = np.empty((D, D), dtype=np.float64)
    if _load().vo_hadamard(D, _dp(H)) != 0:
        raise ValueError("D must be a power of two")
    return H


def smoothing_factors(K) -> np.ndarray:
    """Eq. 4: lambda_i = sqrt(max_n |K[n, i]|) over all rows of K [..., D]."""
    K = _f64(K)
    D = K.shape[-1]
    K2 = K.reshape(-1, D)
    lam = np.empty(D, dtype=np.float64)
    _load().vo_smoothing_factors(_dp(K2), K2.shape[0], D, _dp(lam))
    return lam


def transform_keys(K, lam) -> np.ndarray:
    """K diag(lam)^-1 H_D for K [N, D] (Eq. 3 and Eq. 6, key side)."""
    K = _f64(K)
    lam = _f64(lam)
    N, D = K.shape
    H = hadamard(D)
    out = np.empty_like(K)
    _load().vo_transform_keys(_dp(K), N, D, _dp(lam), _dp(H), _dp(out))
    return out


def transform_query(q, lam) -> np.ndarray:
    """q diag(lam) H_D for one query row q [D] (Eq. 3 and Eq. 6, query side)."""
    q = _f64(q)
    lam = _f64(lam)
    D = q.shape[0]
    H = hadamard(D)
    out = np.empty_like(q)
    _load().vo_transform_query(_dp(q), D, _dp(lam), _dp(H), _dp(out))
    return out


def vq_encode(X, cb, want_gap: bool = False):
    """Eq. 2 on rows X [N, D] with per-sub-space codebooks cb [M, C, d]."""
    X = _f64(X)
    cb = _f64(cb)
    N, D = X.shape
    M, Cn, d = cb.shape
    if M * d != D or Cn > 256:
        # shared codebook ([1, C, d]) and / or more than 256 centroids: uint16 indices
        assert M == 1 or M * d == D
        idx = np.empty((N, D // d), dtype=np.uint16)
        gap = np.empty((N, D // d), dtype=np.float64) if want_gap else None
        _load().vo_vq_encode_g(_dp(X), N, D, d, Cn, M, _dp(cb), _u16p(idx), _dp(gap) if want_gap else None)
        return (idx, gap) if want_gap else idx
    assert M * d == D
    idx = np.empty((N, M), dtype=np.uint8)
    gap = np.empty((N, M), dtype=np.float64) if want_gap else None
    _load().vo_vq_encode(_dp(X), N, D, d, Cn, _dp(cb), _u8p(idx), _dp(gap) if want_gap else None)
    return (idx, gap) if want_gap else idx


def vq_dequantize(idx, cb) -> np.ndarray:
    """VQ^{-1}: rows of concatenated centroids, idx [N, M], cb [M, C, d] -> [N, D]."""
    cb = _f64(cb)
    N, M = np.asarray(idx).shape
    M2, Cn, d = cb.shape
    if M2 != M or Cn > 256:
        assert M2 in (1, M)
        idx = np.ascontiguousarray(idx, dtype=np.uint16)
        assert int(idx.max(initial=0)) < Cn
        out = np.empty((N, M * d), dtype=np.float64)
        _load().vo_vq_dequantize_g(_u16p(idx), N, M * d, d, Cn, M2, _dp(cb), _dp(out))
        return out
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    assert M == M2
    out = np.empty((N, M * d), dtype=np.float64)
    _load().vo_vq_dequantize(_u8p(idx), N, M * d, d, Cn, _dp(cb), _dp(out))
    return out


def merge_splits(o_parts, L_parts):
    """LSE merge of S partial (o, L) pairs of one query row."""
    o_parts = _f64(o_parts)
    L_parts = _f64(L_parts)
    S, D = o_parts.shape
    out = np.empty(D, dtype=np.float64)
    lse = C.c_double()
    _load().vo_merge_splits(_dp(o_parts), _dp(L_parts), S, D, _dp(out), C.byref(lse))
    return out, float(lse.value)


def encode_keys(k_f16, lam, cb_k, want_gap: bool = False):
    """Smooth + Hadamard + VQ of keys (Alg. 1 steps 2-3, Eq. 8).

    k_f16 [B, Hkv, T, D], lam [Hkv, D], cb_k [Hkv, M, C, d] -> uint8 [B, Hkv, T, M].
    """
    return _encode(k_f16, lam, cb_k, 1, want_gap)


def encode_values(v_f16, cb_v, want_gap: bool = False):
    """VQ of the untransformed values (Eq. 8): [B, Hkv, T, D] -> uint8 [B, Hkv, T, M]."""
    return _encode(v_f16, None, cb_v, 0, want_gap)


def _encode(x, lam, cb, transform, want_gap):
    x = _f64(x)
    cb = _f64(cb)
    B, Hkv, T, D = x.shape
    Hc, M, Cn, d = cb.shape
    if M * d != D or Cn > 256:
        return _encode_g(x, lam, cb, transform, want_gap)
    assert Hc == Hkv and M * d == D
    lam64 = _f64(lam) if transform else np.ones((Hkv, D), dtype=np.float64)
    assert lam64.shape == (Hkv, D)
    idx = np.empty((B, Hkv, T, M), dtype=np.uint8)
    gap = np.empty((B, Hkv, T, M), dtype=np.float64) if want_gap else None
    rc = _load().vo_encode_batch(_dp(x), _dp(lam64), _dp(cb), B, Hkv, T, D, d, Cn, transform,
                                 _u8p(idx), _dp(gap) if want_gap else None)
    if rc != 0:
        raise ValueError("vo_encode_batch rejected the shapes")
    return (idx, gap) if want_gap else idx


def _encode_g(x, lam, cb, transform, want_gap):
    """General encode: cb [Hkv, Mcb, C, d] with Mcb = D / d (per sub-space) or 1 (one codebook shared by
    the sub-spaces of a head, the form of Alg. 1 and Sec. 2.2), C up to 65536 -> uint16 [B, Hkv, T, M]."""
    B, Hkv, T, D = x.shape
    Hc, Mcb, Cn, d = cb.shape
    M = D // d
    assert Hc == Hkv and M * d == D and Mcb in (1, M)
    lam64 = _f64(lam) if transform else np.ones((Hkv, D), dtype=np.float64)
    assert lam64.shape == (Hkv, D)
    idx = np.empty((B, Hkv, T, M), dtype=np.uint16)
    gap = np.empty((B, Hkv, T, M), dtype=np.float64) if want_gap else None
    rc = _load().vo_encode_batch_g(_dp(x), _dp(lam64), _dp(cb), B, Hkv, T, D, d, Cn, Mcb, transform,
                                   _u16p(idx), _dp(gap) if want_gap else None)
    if rc != 0:
        raise ValueError("vo_encode_batch_g rejected the shapes")
    return (idx, gap) if want_gap else idx


def pack_codes(idx, bits: int) -> np.ndarray:
    """Rows of M codes of `bits` bits each -> rows of M * bits / 8 bytes: the codes laid end to end
    as one little-endian bit string (code m fills bits m * bits .. (m + 1) * bits - 1 of the row;
    bit i of the row is bit i % 8 of byte i // 8).  This is the "(d_h / d) x (b / 8) bytes for the
    indices" of Sec. 2.2.  idx [..., M] unsigned, every value < 2^bits."""
    idx = np.asarray(idx)
    M = idx.shape[-1]
    assert (M * bits) % 8 == 0 and int(idx.max(initial=0)) < (1 << bits)
    one = ((idx[..., None].astype(np.uint32) >> np.arange(bits, dtype=np.uint32)) & 1).astype(np.uint8)
    return np.packbits(one.reshape(*idx.shape[:-1], M * bits), axis=-1, bitorder="little")


def unpack_codes(packed, bits: int, M: int) -> np.ndarray:
    """Inverse of pack_codes: uint8 [..., M * bits / 8] -> uint16 [..., M]."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.shape[-1] * 8 == M * bits
    one = np.unpackbits(packed, axis=-1, bitorder="little").reshape(*packed.shape[:-1], M, bits)
    out = np.zeros(one.shape[:-1], dtype=np.uint16)
    for i in range(bits):
        out |= one[..., i].astype(np.uint16) << np.uint16(i)
    return out


def _decode_g(q, lam, cb_k, cb_v, k_idx, v_idx, seq_lens):
    B, Hq, D = q.shape
    Hkv, Mcb_k, C_k, d_k = cb_k.shape
    _, Mcb_v, C_v, d_v = cb_v.shape
    Mk, Mv = D // d_k, D // d_v
    k_idx = np.ascontiguousarray(k_idx, dtype=np.uint16)
    v_idx = np.ascontiguousarray(v_idx, dtype=np.uint16)
    assert Mcb_k in (1, Mk) and Mcb_v in (1, Mv)
    assert k_idx.shape[:2] == (B, Hkv) and k_idx.shape[3] == Mk and v_idx.shape[3] == Mv
    assert int(k_idx.max(initial=0)) < C_k and int(v_idx.max(initial=0)) < C_v
    n_cap = k_idx.shape[2]
    sl = np.full(B, n_cap, dtype=np.int64) if seq_lens is None else np.ascontiguousarray(seq_lens, dtype=np.int64)
    assert sl.shape == (B,) and int(sl.max()) <= n_cap
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    rc = _load().vo_decode_batch_g(_dp(q), _dp(lam), _dp(cb_k), _dp(cb_v), _u16p(k_idx), _u16p(v_idx),
                                   sl.ctypes.data_as(C.POINTER(C.c_int64)), B, Hq, Hkv, n_cap, D, d_k, C_k, Mcb_k,
                                   d_v, C_v, Mcb_v, _dp(out), _dp(lse))
    if rc != 0:
        raise ValueError("vo_decode_batch_g rejected the inputs (empty sequence or bad shapes)")
    return out, lse


def decode_attention(q_f16, lam, cb_k, cb_v, k_idx, v_idx, seq_lens=None, *,
                     path: str = "eq10", tile: int = 64):
    """One decode step of VQ attention for a batch (Eq. 10; GQA by consecutive groups).

    q_f16 [B, Hq, D]; lam [Hkv, D]; cb_k [Hkv, Mk, C, d_k]; cb_v [Hkv, Mv, C, d_v];
    k_idx [B, Hkv, n_cap, Mk]; v_idx [B, Hkv, n_cap, Mv]; seq_lens [B] or None (= n_cap).
    path "eq10": explicit dequantize-then-attend; "alg1": lookup table + online softmax
    over tiles of `tile` tokens.  Returns (out [B, Hq, D] f64, lse [B, Hq] f64).

    A codebook may also be [Hkv, 1, C, d] (shared by the sub-spaces of a head) and C may exceed
    256, with unpacked uint16 indices; keys and values may then differ in C (path "eq10" only).
    """
    q = _f64(q_f16)
    lam = _f64(lam)
    cb_k = _f64(cb_k)
    cb_v = _f64(cb_v)
    if (cb_k.shape[1] * cb_k.shape[3] != q.shape[2] or cb_v.shape[1] * cb_v.shape[3] != q.shape[2]
            or cb_k.shape[2] > 256 or cb_v.shape[2] > 256):
        assert path == "eq10"
        return _decode_g(q, lam, cb_k, cb_v, k_idx, v_idx, seq_lens)
    k_idx = np.ascontiguousarray(k_idx, dtype=np.uint8)
    v_idx = np.ascontiguousarray(v_idx, dtype=np.uint8)
    B, Hq, D = q.shape
    Hkv, Mk, Cn, d_k = cb_k.shape
    _, Mv, Cv, d_v = cb_v.shape
    assert Cn == Cv and k_idx.shape[:2] == (B, Hkv) and v_idx.shape[:2] == (B, Hkv)
    assert k_idx.shape[3] == Mk and v_idx.shape[3] == Mv and k_idx.shape[2] == v_idx.shape[2]
    n_cap = k_idx.shape[2]
    if seq_lens is None:
        sl = np.full(B, n_cap, dtype=np.int64)
    else:
        sl = np.ascontiguousarray(seq_lens, dtype=np.int64)
    assert sl.shape == (B,) and int(sl.max()) <= n_cap
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    rc = _load().vo_decode_batch(_dp(q), _dp(lam), _dp(cb_k), _dp(cb_v), _u8p(k_idx), _u8p(v_idx),
                                 sl.ctypes.data_as(C.POINTER(C.c_int64)), B, Hq, Hkv, n_cap, D,
                                 d_k, d_v, Cn, {"eq10": 0, "alg1": 1}[path], int(tile),
                                 _dp(out), _dp(lse))
    if rc != 0:
        raise ValueError("vo_decode_batch rejected the inputs (empty sequence or bad shapes)")
    return out, lse


def decode_attention_residual(q_f16, lam, cb_k, cb_v, k_idx, v_idx, k_res, v_res, seq_lens=None, res_lens=None):
    """Decode step with a full-precision residual window (Sec. 4.1, residual length):
    Eq. 10 over the quantized tokens plus raw-query x raw-key scores for the window, one
    softmax over both.  k_res, v_res [B, Hkv, r_cap, D] (fp16 in the GPU path); res_lens [B]
    or None (= r_cap).  seq_lens[b] may be 0 if the window of b is not empty.
    Returns (out [B, Hq, D] f64, lse [B, Hq] f64)."""
    q = _f64(q_f16)
    lam = _f64(lam)
    cb_k = _f64(cb_k)
    cb_v = _f64(cb_v)
    k_res = _f64(k_res)
    v_res = _f64(v_res)
    B, Hq, D = q.shape
    Hkv, Mk, Cn, d_k = cb_k.shape
    _, Mv, Cv, d_v = cb_v.shape
    n_cap = np.asarray(k_idx).shape[2]
    r_cap = k_res.shape[2]
    assert k_res.shape == (B, Hkv, r_cap, D) and v_res.shape == (B, Hkv, r_cap, D)
    sl = np.full(B, n_cap, dtype=np.int64) if seq_lens is None else np.ascontiguousarray(seq_lens, dtype=np.int64)
    rl = np.full(B, r_cap, dtype=np.int64) if res_lens is None else np.ascontiguousarray(res_lens, dtype=np.int64)
    assert int(sl.max()) <= n_cap and int(rl.max()) <= r_cap
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    i64p = C.POINTER(C.c_int64)
    if Mk * d_k != D or Mv * d_v != D or Cn > 256 or Cv > 256:
        # shared codebooks ([Hkv, 1, C, d]) and / or more than 256 centroids: unpacked uint16 indices
        k16 = np.ascontiguousarray(k_idx, dtype=np.uint16)
        v16 = np.ascontiguousarray(v_idx, dtype=np.uint16)
        assert Mk in (1, D // d_k) and Mv in (1, D // d_v)
        assert k16.shape == (B, Hkv, n_cap, D // d_k) and v16.shape == (B, Hkv, n_cap, D // d_v)
        assert int(k16.max(initial=0)) < Cn and int(v16.max(initial=0)) < Cv
        rc = _load().vo_decode_residual_batch_g(_dp(q), _dp(lam), _dp(cb_k), _dp(cb_v), _u16p(k16), _u16p(v16),
                                                sl.ctypes.data_as(i64p), _dp(k_res), _dp(v_res),
                                                rl.ctypes.data_as(i64p), B, Hq, Hkv, n_cap, r_cap, D, d_k, Cn, Mk,
                                                d_v, Cv, Mv, _dp(out), _dp(lse))
        if rc != 0:
            raise ValueError("vo_decode_residual_batch_g rejected the inputs")
        return out, lse
    k_idx = np.ascontiguousarray(k_idx, dtype=np.uint8)
    v_idx = np.ascontiguousarray(v_idx, dtype=np.uint8)
    rc = _load().vo_decode_residual_batch(_dp(q), _dp(lam), _dp(cb_k), _dp(cb_v), _u8p(k_idx), _u8p(v_idx),
                                          sl.ctypes.data_as(i64p), _dp(k_res), _dp(v_res), rl.ctypes.data_as(i64p),
                                          B, Hq, Hkv, n_cap, r_cap, D, d_k, d_v, Cn, _dp(out), _dp(lse))
    if rc != 0:
        raise ValueError("vo_decode_residual_batch rejected the inputs (a sequence with no token at all, or bad shapes)")
    return out, lse


def kmeans_update(X, idx, cb_in):
    """Centroid update of one Lloyd iteration of the K-Means codebook training (Sec. 2.2, 4.1):
    X [N, D] rows (keys already transformed), idx [N, M] their codes, cb_in [M, C, d].
    Returns (cb_out [M, C, d] f64, counts [M, C] int64); an empty cluster keeps its centroid."""
    X = _f64(X)
    cb_in = _f64(cb_in)
    N, D = X.shape
    M, Cn, d = cb_in.shape
    if M * d != D or Cn > 256:
        # one codebook shared by the sub-spaces ([1, C, d]): trained on their sub-vectors pooled
        assert M in (1, D // d)
        idx = np.ascontiguousarray(idx, dtype=np.uint16)
        assert idx.shape == (N, D // d) and int(idx.max(initial=0)) < Cn
        cb_out = np.empty_like(cb_in)
        counts = np.empty((M, Cn), dtype=np.int64)
        _load().vo_kmeans_update_g(_dp(X), _u16p(idx), N, D, d, Cn, M, _dp(cb_in), _dp(cb_out),
                                   counts.ctypes.data_as(C.POINTER(C.c_int64)))
        return cb_out, counts
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    assert M * d == D and idx.shape == (N, M)
    cb_out = np.empty_like(cb_in)
    counts = np.empty((M, Cn), dtype=np.int64)
    _load().vo_kmeans_update(_dp(X), _u8p(idx), N, D, d, Cn, _dp(cb_in), _dp(cb_out),
                             counts.ctypes.data_as(C.POINTER(C.c_int64)))
    return cb_out, counts


def kmeans_step(x_f16, lam, cb):
    """One Lloyd iteration per (KV head, sub-space) over all tokens of all sequences:
    x_f16 [B, Hkv, T, D]; lam [Hkv, D] (keys: trained on the transformed keys, Sec. 3.2) or None
    (values: raw); cb [Hkv, M, C, d], or [Hkv, 1, C, d] for a codebook shared by the sub-spaces.
    Returns (cb_new like cb, f64; counts [Hkv, M or 1, C]; idx [B, Hkv, T, M])."""
    x = _f64(x_f16)
    cb = _f64(cb)
    B, Hkv, T, D = x.shape
    idx = encode_keys(x_f16, lam, cb) if lam is not None else encode_values(x_f16, cb)
    cb_new = np.empty_like(cb)
    counts = np.empty(cb.shape[:3], dtype=np.int64)
    for g in range(Hkv):
        rows = x[:, g].reshape(B * T, D)
        if lam is not None:
            rows = transform_keys(rows, _f64(lam)[g])
        cb_new[g], counts[g] = kmeans_update(rows, idx[:, g].reshape(B * T, -1), cb[g])
    return cb_new, counts, idx


def quantization_error(x_f16, lam, cb, idx):
    """Sum over all sub-vectors of the squared distance to the centroid they are coded with (the
    K-Means objective, Sec. 2.2): x_f16 [B, Hkv, T, D]; lam [Hkv, D] or None (values); cb
    [Hkv, M, C, d] (or [Hkv, 1, C, d], shared); idx [B, Hkv, T, M].  Returns one float per KV head."""
    x = _f64(x_f16)
    cb = _f64(cb)
    B, Hkv, T, D = x.shape
    err = np.zeros(Hkv)
    for g in range(Hkv):
        rows = x[:, g].reshape(B * T, D)
        if lam is not None:
            rows = transform_keys(rows, _f64(lam)[g])
        err[g] = ((rows - vq_dequantize(idx[:, g].reshape(B * T, -1), cb[g])) ** 2).sum()
    return err


def kmeans_train(x_f16, lam, cb0, max_iters=30, tol=1e-4, round_f16=True):
    """K-Means codebook training (Sec. 2.2; Sec. 3.2: on the transformed keys / the original values;
    Sec. 4.1: at most 30 iterations), Lloyd's algorithm as a loop of kmeans_step.
    Iteration t assigns every sub-vector to its nearest centroid of cb_t (Eq. 2), records the
    quantization error E_t of that assignment (all KV heads together), and replaces every centroid
    by the mean of its cluster (an empty cluster keeps its centroid) -> cb_{t+1}.  The loop stops
    after the update of iteration t when t = max_iters - 1, or when t >= 1 and
    E_{t-1} - E_t <= tol * E_{t-1} (the improvement has died down; a negative tol never stops early).
    round_f16: the codebook is stored in fp16 (2 bytes per element, Sec. 2.2), so each cb_{t+1} is
    rounded to fp16 before the next assignment.
    Returns (cb [like cb0, f64], counts and idx of the last assignment, errors [iterations run])."""
    cb = _f64(cb0)
    errors = []
    counts = idx = None
    for t in range(max_iters):
        cb_new, counts, idx = kmeans_step(x_f16, lam, cb)
        errors.append(float(quantization_error(x_f16, lam, cb, idx).sum()))
        cb = _f64(cb_new.astype(np.float16)) if round_f16 else cb_new
        if t >= 1 and errors[t - 1] - errors[t] <= tol * errors[t - 1]:
            break
    return cb, counts, idx, np.array(errors)
