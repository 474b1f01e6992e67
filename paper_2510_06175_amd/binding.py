"""ctypes binding of ``libvecinfer.so``: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA (HIP) tensors used purely as device buffers; shapes, dtypes,
contiguity and device are checked here and the raw pointers handed to the library,
which enqueues on torch's current stream unless ``stream`` is given.  If the library
has not been built the import of it fails loudly: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvecinfer.so")

VARIANT_AUTO, VARIANT_LUT, VARIANT_MFMA, VARIANT_ROLES = 0, 1, 2, 3
MAX_SPLITS = 256
MAX_RESIDUAL = 128
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, ELAUNCH = 0, -1, -2, -3, -4

EXPORTS = [
    "vecinfer_encode_keys", "vecinfer_encode_values", "vecinfer_append_kv", "vecinfer_decode_auto_splits",
    "vecinfer_decode_workspace_bytes",
    "vecinfer_decode_attention", "vecinfer_decode_attention_residual", "vecinfer_decode_step",
    "vecinfer_decode_attention_static",
    "vecinfer_kmeans_workspace_bytes", "vecinfer_kmeans_step", "vecinfer_kmeans_train",
    "vecinfer_index_row_bytes", "vecinfer_codebook_elems", "vecinfer_calibrate_lambda", "vecinfer_read_probe",
    "vecinfer_export_value_codes",
    "vecinfer_strerror", "vecinfer_version",
]


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("head_dim", "num_q_heads", "num_kv_heads", "k_sub_dim",
                                         "v_sub_dim", "k_bits", "v_bits", "v_tiled")]


@dataclass(frozen=True)
class Config:
    """Mirror of ``vecinfer_cfg``."""
    head_dim: int
    num_q_heads: int
    num_kv_heads: int
    k_sub_dim: int
    v_sub_dim: int
    k_bits: int = 8
    v_bits: int = 8
    v_tiled: int = 0            # 1: value codes stored in tiles of 64 tokens (8-bit value codes)

    def c(self) -> _Cfg:
        return _Cfg(self.head_dim, self.num_q_heads, self.num_kv_heads, self.k_sub_dim,
                    self.v_sub_dim, self.k_bits, self.v_bits, self.v_tiled)

    def cb_shape(self, keys: bool) -> tuple:
        """Codebook tensor shape: one 256-entry table per (KV head, sub-space) for 8-bit codes, one
        table of 2^bits entries per KV head for wider ones."""
        d, bits = (self.k_sub_dim, self.k_bits) if keys else (self.v_sub_dim, self.v_bits)
        if bits == 8:
            return (self.num_kv_heads, self.head_dim // d, 256, d)
        return (self.num_kv_heads, 1 << bits, d)

    def row_bytes(self, keys: bool) -> int:
        """Bytes of one token's code row: M codes of `bits` bits, end to end."""
        d, bits = (self.k_sub_dim, self.k_bits) if keys else (self.v_sub_dim, self.v_bits)
        return self.head_dim // d * bits // 8


class VecInferError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"vecinfer error {code}: {strerror(code)}")


_lib = None


def lib() -> C.CDLL:
    """Load the built library (raises if it is missing: build it first)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -m paper_2510_06175_amd.build` "
                "(or __graft_entry__.build()) first")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        cfgp = C.POINTER(_Cfg)
        L.vecinfer_encode_keys.argtypes = [cfgp, vp, vp, vp, vp, i32, i64, i64, i64, vp]
        L.vecinfer_encode_keys.restype = C.c_int
        L.vecinfer_encode_values.argtypes = [cfgp, vp, vp, vp, i32, i64, i64, i64, vp]
        L.vecinfer_encode_values.restype = C.c_int
        L.vecinfer_append_kv.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, i32, i64, i64, i64, vp]
        L.vecinfer_append_kv.restype = C.c_int
        L.vecinfer_decode_auto_splits.argtypes = [cfgp, i32, i64]
        L.vecinfer_decode_auto_splits.restype = i32
        L.vecinfer_decode_workspace_bytes.argtypes = [cfgp, i32, i64, i32]
        L.vecinfer_decode_workspace_bytes.restype = sz
        L.vecinfer_decode_attention.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, i32, i64, i64, i32,
                                                i32, vp, sz, vp, vp, vp]
        L.vecinfer_decode_attention.restype = C.c_int
        L.vecinfer_decode_attention_static.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, i32, i64, i64, i32,
                                                       i32, vp, vp, vp]
        L.vecinfer_decode_attention_static.restype = C.c_int
        L.vecinfer_decode_attention_residual.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, i32, i64, i64, vp, vp,
                                                         vp, i32, i64, i32, i32, vp, sz, vp, vp, vp]
        L.vecinfer_decode_attention_residual.restype = C.c_int
        L.vecinfer_decode_step.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i64, i64, i32, i32, vp, sz,
                                           vp, vp, vp]
        L.vecinfer_decode_step.restype = C.c_int
        L.vecinfer_kmeans_workspace_bytes.argtypes = [cfgp, i32]
        L.vecinfer_kmeans_workspace_bytes.restype = sz
        L.vecinfer_kmeans_step.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, i32, i64, vp, sz, vp]
        L.vecinfer_kmeans_step.restype = C.c_int
        L.vecinfer_kmeans_train.argtypes = [cfgp, vp, vp, vp, vp, vp, i32, i64, i32, C.c_float, vp, vp, vp, sz, vp]
        L.vecinfer_kmeans_train.restype = C.c_int
        L.vecinfer_calibrate_lambda.argtypes = [cfgp, vp, vp, i32, i64, vp]
        L.vecinfer_calibrate_lambda.restype = C.c_int
        L.vecinfer_read_probe.argtypes = [vp, sz, vp, vp]
        L.vecinfer_read_probe.restype = C.c_int
        L.vecinfer_export_value_codes.argtypes = [cfgp, vp, vp, i32, i64, i64, vp]
        L.vecinfer_export_value_codes.restype = C.c_int
        L.vecinfer_index_row_bytes.argtypes = [cfgp, i32]
        L.vecinfer_index_row_bytes.restype = sz
        L.vecinfer_codebook_elems.argtypes = [cfgp, i32]
        L.vecinfer_codebook_elems.restype = sz
        L.vecinfer_strerror.argtypes = [C.c_int]
        L.vecinfer_strerror.restype = C.c_char_p
        L.vecinfer_version.restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().vecinfer_strerror(int(code)).decode()


def vecinfer_version() -> int:
    return int(lib().vecinfer_version())


def _check(rc: int) -> None:
    if rc != 0:
        raise VecInferError(rc)


def _dev(t: torch.Tensor, dtype, shape, name: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a tensor on the GPU")
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
        raise ValueError(f"{name}: expected contiguous {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def vecinfer_encode_keys(cfg: Config, k_f16, lam, cb_k, k_idx, pos0: int = 0, stream=None) -> None:
    """Smooth + Hadamard + VQ of T new keys into rows pos0.. of the code cache."""
    B, Hkv, T, D = k_f16.shape
    n_cap = k_idx.shape[2]
    _check(lib().vecinfer_encode_keys(
        C.byref(cfg.c()), _dev(k_f16, torch.float16, (B, cfg.num_kv_heads, T, cfg.head_dim), "k_f16"),
        _dev(lam, torch.float32, (cfg.num_kv_heads, cfg.head_dim), "lambda"),
        _dev(cb_k, torch.float16, cfg.cb_shape(True), "cb_k"),
        _dev(k_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(True)), "k_idx"),
        B, T, pos0, n_cap, _stream(stream)))


def vecinfer_encode_values(cfg: Config, v_f16, cb_v, v_idx, pos0: int = 0, stream=None) -> None:
    """VQ of T new (untransformed) values into rows pos0.. of the code cache."""
    B, Hkv, T, D = v_f16.shape
    n_cap = v_idx.shape[2]
    _check(lib().vecinfer_encode_values(
        C.byref(cfg.c()), _dev(v_f16, torch.float16, (B, cfg.num_kv_heads, T, cfg.head_dim), "v_f16"),
        _dev(cb_v, torch.float16, cfg.cb_shape(False), "cb_v"),
        _dev(v_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(False)), "v_idx"),
        B, T, pos0, n_cap, _stream(stream)))


def vecinfer_append_kv(cfg: Config, k_f16, v_f16, lam, cb_k, cb_v, k_idx, v_idx, pos0: int, stream=None) -> None:
    """Decode-time append (Eq. 9): encode T <= 16 new keys and values in one launch."""
    B, Hkv, T, D = k_f16.shape
    n_cap = k_idx.shape[2]
    _check(lib().vecinfer_append_kv(
        C.byref(cfg.c()), _dev(k_f16, torch.float16, (B, cfg.num_kv_heads, T, cfg.head_dim), "k_f16"),
        _dev(v_f16, torch.float16, (B, cfg.num_kv_heads, T, cfg.head_dim), "v_f16"),
        _dev(lam, torch.float32, (cfg.num_kv_heads, cfg.head_dim), "lambda"),
        _dev(cb_k, torch.float16, cfg.cb_shape(True), "cb_k"),
        _dev(cb_v, torch.float16, cfg.cb_shape(False), "cb_v"),
        _dev(k_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(True)), "k_idx"),
        _dev(v_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(False)), "v_idx"),
        B, T, pos0, n_cap, _stream(stream)))


def vecinfer_decode_auto_splits(cfg: Config, B: int, N: int) -> int:
    return int(lib().vecinfer_decode_auto_splits(C.byref(cfg.c()), B, N))


def vecinfer_decode_workspace_bytes(cfg: Config, B: int, N: int, num_splits: int = 0) -> int:
    return int(lib().vecinfer_decode_workspace_bytes(C.byref(cfg.c()), B, N, num_splits))


def new_workspace(cfg: Config, B: int, N: int, num_splits: int = 0, device="cuda") -> torch.Tensor:
    """Allocate (with torch) a workspace for vecinfer_decode_attention."""
    nbytes = vecinfer_decode_workspace_bytes(cfg, B, N, num_splits)
    if nbytes == 0:
        raise VecInferError(EUNSUPPORTED)
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def vecinfer_decode_attention(cfg: Config, q_f16, lam, cb_k, cb_v, k_idx, v_idx, workspace, out_f16,
                              lse=None, seq_lens=None, N: int | None = None, num_splits: int = 0,
                              variant: int = VARIANT_AUTO, stream=None) -> None:
    """One fused VQ decode-attention step; writes out_f16 [B, Hq, D] (and lse [B, Hq])."""
    B = q_f16.shape[0]
    n_cap = k_idx.shape[2]
    N = n_cap if N is None else N
    _check(lib().vecinfer_decode_attention(
        C.byref(cfg.c()), _dev(q_f16, torch.float16, (B, cfg.num_q_heads, cfg.head_dim), "q_f16"),
        _dev(lam, torch.float32, (cfg.num_kv_heads, cfg.head_dim), "lambda"),
        _dev(cb_k, torch.float16, cfg.cb_shape(True), "cb_k"),
        _dev(cb_v, torch.float16, cfg.cb_shape(False), "cb_v"),
        _dev(k_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(True)), "k_idx"),
        _dev(v_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(False)), "v_idx"),
        None if seq_lens is None else _dev(seq_lens, torch.int32, (B,), "seq_lens"),
        B, N, n_cap, num_splits, variant, workspace.data_ptr(), workspace.numel() * workspace.element_size(),
        _dev(out_f16, torch.float16, (B, cfg.num_q_heads, cfg.head_dim), "out_f16"),
        None if lse is None else _dev(lse, torch.float32, (B, cfg.num_q_heads), "lse"),
        _stream(stream)))


STATIC_SCRATCH_BYTES = 4 << 20


def vecinfer_decode_attention_static(cfg: Config, q_f16, lam, cb_k, cb_v, k_idx, v_idx, out_f16,
                                     lse=None, seq_lens=None, N: int | None = None, num_splits: int = 0,
                                     variant: int = VARIANT_AUTO, stream=None) -> None:
    """vecinfer_decode_attention without a workspace argument: the split partials live in a fixed
    array inside the library (STATIC_SCRATCH_BYTES per GPU); the call allocates nothing."""
    B = q_f16.shape[0]
    n_cap = k_idx.shape[2]
    N = n_cap if N is None else N
    _check(lib().vecinfer_decode_attention_static(
        C.byref(cfg.c()), _dev(q_f16, torch.float16, (B, cfg.num_q_heads, cfg.head_dim), "q_f16"),
        _dev(lam, torch.float32, (cfg.num_kv_heads, cfg.head_dim), "lambda"),
        _dev(cb_k, torch.float16, cfg.cb_shape(True), "cb_k"),
        _dev(cb_v, torch.float16, cfg.cb_shape(False), "cb_v"),
        _dev(k_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(True)), "k_idx"),
        _dev(v_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(False)), "v_idx"),
        None if seq_lens is None else _dev(seq_lens, torch.int32, (B,), "seq_lens"),
        B, N, n_cap, num_splits, variant,
        _dev(out_f16, torch.float16, (B, cfg.num_q_heads, cfg.head_dim), "out_f16"),
        None if lse is None else _dev(lse, torch.float32, (B, cfg.num_q_heads), "lse"),
        _stream(stream)))


def vecinfer_decode_attention_residual(cfg: Config, q_f16, lam, cb_k, cb_v, k_idx, v_idx, k_res, v_res, workspace,
                                       out_f16, lse=None, seq_lens=None, res_lens=None, N: int | None = None,
                                       R: int | None = None, num_splits: int = 0, variant: int = VARIANT_AUTO,
                                       stream=None) -> None:
    """Decode step over the code cache plus a full-precision window k_res / v_res [B, Hkv, r_cap, D]."""
    B = q_f16.shape[0]
    n_cap = k_idx.shape[2]
    N = n_cap if N is None else N
    r_cap = k_res.shape[2]
    R = r_cap if R is None else R
    _check(lib().vecinfer_decode_attention_residual(
        C.byref(cfg.c()), _dev(q_f16, torch.float16, (B, cfg.num_q_heads, cfg.head_dim), "q_f16"),
        _dev(lam, torch.float32, (cfg.num_kv_heads, cfg.head_dim), "lambda"),
        _dev(cb_k, torch.float16, cfg.cb_shape(True), "cb_k"),
        _dev(cb_v, torch.float16, cfg.cb_shape(False), "cb_v"),
        _dev(k_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(True)), "k_idx"),
        _dev(v_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(False)), "v_idx"),
        None if seq_lens is None else _dev(seq_lens, torch.int32, (B,), "seq_lens"),
        B, N, n_cap,
        _dev(k_res, torch.float16, (B, cfg.num_kv_heads, r_cap, cfg.head_dim), "k_res"),
        _dev(v_res, torch.float16, (B, cfg.num_kv_heads, r_cap, cfg.head_dim), "v_res"),
        None if res_lens is None else _dev(res_lens, torch.int32, (B,), "res_lens"),
        R, r_cap, num_splits, variant, workspace.data_ptr(), workspace.numel() * workspace.element_size(),
        _dev(out_f16, torch.float16, (B, cfg.num_q_heads, cfg.head_dim), "out_f16"),
        None if lse is None else _dev(lse, torch.float32, (B, cfg.num_q_heads), "lse"),
        _stream(stream)))


def vecinfer_decode_step(cfg: Config, q_f16, k_new, v_new, lam, cb_k, cb_v, k_idx, v_idx, workspace, out_f16,
                         lse=None, seq_lens=None, N: int | None = None, num_splits: int = 0,
                         variant: int = VARIANT_AUTO, stream=None) -> None:
    """Append the new token (k_new, v_new [B, Hkv, 1, D]) as each sequence's last one and attend."""
    B = q_f16.shape[0]
    n_cap = k_idx.shape[2]
    N = n_cap if N is None else N
    _check(lib().vecinfer_decode_step(
        C.byref(cfg.c()), _dev(q_f16, torch.float16, (B, cfg.num_q_heads, cfg.head_dim), "q_f16"),
        _dev(k_new, torch.float16, (B, cfg.num_kv_heads, 1, cfg.head_dim), "k_new"),
        _dev(v_new, torch.float16, (B, cfg.num_kv_heads, 1, cfg.head_dim), "v_new"),
        _dev(lam, torch.float32, (cfg.num_kv_heads, cfg.head_dim), "lambda"),
        _dev(cb_k, torch.float16, cfg.cb_shape(True), "cb_k"),
        _dev(cb_v, torch.float16, cfg.cb_shape(False), "cb_v"),
        _dev(k_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(True)), "k_idx"),
        _dev(v_idx, torch.uint8, (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(False)), "v_idx"),
        None if seq_lens is None else _dev(seq_lens, torch.int32, (B,), "seq_lens"),
        B, N, n_cap, num_splits, variant, workspace.data_ptr(), workspace.numel() * workspace.element_size(),
        _dev(out_f16, torch.float16, (B, cfg.num_q_heads, cfg.head_dim), "out_f16"),
        None if lse is None else _dev(lse, torch.float32, (B, cfg.num_q_heads), "lse"),
        _stream(stream)))


def vecinfer_index_row_bytes(cfg: Config, keys: bool) -> int:
    return int(lib().vecinfer_index_row_bytes(C.byref(cfg.c()), 1 if keys else 0))


def vecinfer_codebook_elems(cfg: Config, keys: bool) -> int:
    return int(lib().vecinfer_codebook_elems(C.byref(cfg.c()), 1 if keys else 0))


LAMBDA_FLOOR = 1e-5


def vecinfer_calibrate_lambda(cfg: Config, k_f16, lam, stream=None) -> None:
    """Eq. 4: lam [Hkv, D] = sqrt(max |k|) over all tokens of k_f16 [B, Hkv, T, D], floored at LAMBDA_FLOOR."""
    B, Hkv, T, D = k_f16.shape
    _check(lib().vecinfer_calibrate_lambda(
        C.byref(cfg.c()), _dev(k_f16, torch.float16, (B, cfg.num_kv_heads, T, cfg.head_dim), "k_f16"),
        _dev(lam, torch.float32, (cfg.num_kv_heads, cfg.head_dim), "lambda"), B, T, _stream(stream)))


def vecinfer_export_value_codes(cfg: Config, v_idx_tiled, v_idx_rows, N: int | None = None, stream=None) -> None:
    """Rows form [B, Hkv, n_cap, M_v] (rows 0 .. N-1) of a value code cache kept in the tiled layout."""
    B, n_cap = v_idx_rows.shape[0], v_idx_rows.shape[2]
    shape = (B, cfg.num_kv_heads, n_cap, cfg.row_bytes(False))
    _check(lib().vecinfer_export_value_codes(
        C.byref(cfg.c()), _dev(v_idx_tiled, torch.uint8, shape, "v_idx_tiled"),
        _dev(v_idx_rows, torch.uint8, shape, "v_idx_rows"), B, n_cap if N is None else N, n_cap, _stream(stream)))


def vecinfer_read_probe(src, sink, stream=None) -> None:
    """Plain streaming read of the whole tensor `src` (measurement aid); `sink`: any device tensor of >= 4 bytes."""
    if not src.is_cuda or not sink.is_cuda or not src.is_contiguous():
        raise TypeError("read probe: expected contiguous device tensors")
    _check(lib().vecinfer_read_probe(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                                     _stream(stream)))


def vecinfer_kmeans_workspace_bytes(cfg: Config, keys: bool) -> int:
    return int(lib().vecinfer_kmeans_workspace_bytes(C.byref(cfg.c()), 1 if keys else 0))


def new_kmeans_workspace(cfg: Config, keys: bool, device="cuda") -> torch.Tensor:
    return torch.empty(vecinfer_kmeans_workspace_bytes(cfg, keys), dtype=torch.uint8, device=device)


def vecinfer_kmeans_step(cfg: Config, x_f16, lam, cb_in, cb_out, codes, workspace, counts=None, stream=None) -> None:
    """One Lloyd iteration of the codebook training on x_f16 [B, Hkv, T, D]; lam = None trains a
    value codebook (no transform).  Writes cb_out, codes [B, Hkv, T, row bytes] and, if given, counts
    (one per centroid: the codebook's shape without its last axis)."""
    B, Hkv, T, D = x_f16.shape
    keys = lam is not None
    ws = workspace
    cb_shape = cfg.cb_shape(keys)
    _check(lib().vecinfer_kmeans_step(
        C.byref(cfg.c()), _dev(x_f16, torch.float16, (B, cfg.num_kv_heads, T, cfg.head_dim), "x_f16"),
        None if lam is None else _dev(lam, torch.float32, (cfg.num_kv_heads, cfg.head_dim), "lambda"),
        _dev(cb_in, torch.float16, cb_shape, "cb_in"),
        _dev(cb_out, torch.float16, cb_shape, "cb_out"),
        _dev(codes, torch.uint8, (B, cfg.num_kv_heads, T, cfg.row_bytes(keys)), "codes"),
        None if counts is None else _dev(counts, torch.int32, cb_shape[:-1], "counts"),
        B, T, ws.data_ptr(), ws.numel(), _stream(stream)))


KMEANS_MAX_ITERS = 30


def vecinfer_kmeans_train(cfg: Config, x_f16, lam, cb, codes, workspace, counts=None, max_iters: int = 30,
                          tol: float = 1e-4, iters_run=None, errors=None, stream=None) -> None:
    """K-Means training in place on cb (at most max_iters Lloyd iterations, stopping rule on the device).
    iters_run: int32 device tensor [1] or None; errors: float64 device tensor [max_iters] or None."""
    B, Hkv, T, D = x_f16.shape
    keys = lam is not None
    cb_shape = cfg.cb_shape(keys)
    _check(lib().vecinfer_kmeans_train(
        C.byref(cfg.c()), _dev(x_f16, torch.float16, (B, cfg.num_kv_heads, T, cfg.head_dim), "x_f16"),
        None if lam is None else _dev(lam, torch.float32, (cfg.num_kv_heads, cfg.head_dim), "lambda"),
        _dev(cb, torch.float16, cb_shape, "cb"),
        _dev(codes, torch.uint8, (B, cfg.num_kv_heads, T, cfg.row_bytes(keys)), "codes"),
        None if counts is None else _dev(counts, torch.int32, cb_shape[:-1], "counts"),
        B, T, max_iters, tol,
        None if iters_run is None else _dev(iters_run, torch.int32, (1,), "iters_run"),
        None if errors is None else _dev(errors, torch.float64, (max_iters,), "errors"),
        workspace.data_ptr(), workspace.numel(), _stream(stream)))
