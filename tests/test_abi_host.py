"""Host-side checks of the C-ABI library: it loads, exports every declared symbol, and
rejects bad arguments with error codes before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2510_06175_amd import binding as vb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # non-null, 256-byte aligned; never dereferenced on the host


def declared_functions():
    text = open(os.path.join(ROOT, "include", "vecinfer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vecinfer_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert sorted(names) == sorted(vb.EXPORTS)
    L = vb.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_strerror():
    assert vb.vecinfer_version() == 300
    assert vb.strerror(0) == "ok"
    for code in (vb.EINVAL, vb.EUNSUPPORTED, vb.EWORKSPACE, vb.ELAUNCH):
        assert vb.strerror(code) not in ("ok", "unknown error code")
    assert vb.strerror(-99) == "unknown error code"


CFG = vb.Config(128, 32, 8, 4, 4)


def _enc_keys(cfg=CFG, k=FAKE, lam=FAKE, cb=FAKE, idx=FAKE, B=1, T=4, pos0=0, n_cap=8):
    return vb.lib().vecinfer_encode_keys(C.byref(cfg.c()), k, lam, cb, idx, B, T, pos0, n_cap, None)


def _enc_vals(cfg=CFG, v=FAKE, cb=FAKE, idx=FAKE, B=1, T=4, pos0=0, n_cap=8):
    return vb.lib().vecinfer_encode_values(C.byref(cfg.c()), v, cb, idx, B, T, pos0, n_cap, None)


def test_encode_argument_errors():
    assert _enc_keys(k=None) == vb.EINVAL
    assert _enc_keys(lam=None) == vb.EINVAL
    assert _enc_keys(idx=None) == vb.EINVAL
    assert _enc_keys(B=0) == vb.EINVAL
    assert _enc_keys(T=0) == vb.EINVAL
    assert _enc_keys(pos0=-1) == vb.EINVAL
    assert _enc_keys(T=6, pos0=3, n_cap=8) == vb.EINVAL          # runs past the cache
    assert _enc_keys(k=FAKE + 2) == vb.EINVAL                     # misaligned
    assert _enc_vals(v=None) == vb.EINVAL
    assert _enc_vals(T=9) == vb.EINVAL
    for bad in (vb.Config(96, 32, 8, 4, 4), vb.Config(128, 32, 5, 4, 4), vb.Config(128, 32, 8, 3, 4),
                vb.Config(128, 32, 8, 4, 4, k_bits=16), vb.Config(128, 32, 8, 2, 4, k_bits=12),
                vb.Config(64, 32, 8, 4, 8, v_bits=10), vb.Config(64, 32, 8, 8, 4, k_bits=10), vb.Config(128, 32, 8, 4, 4, k_bits=9), vb.Config(128, 128, 8, 4, 4),
                vb.Config(128, 32, 8, 4, 16)):
        assert _enc_keys(cfg=bad) == vb.EUNSUPPORTED
        assert _enc_vals(cfg=bad) == vb.EUNSUPPORTED


def test_append_argument_errors():
    def app(cfg=CFG, k=FAKE, v=FAKE, lam=FAKE, cbk=FAKE, cbv=FAKE, ki=FAKE, vi=FAKE, B=1, T=1, pos0=7, n_cap=8):
        return vb.lib().vecinfer_append_kv(C.byref(cfg.c()), k, v, lam, cbk, cbv, ki, vi, B, T, pos0, n_cap, None)
    assert app(k=None) == vb.EINVAL
    assert app(v=None) == vb.EINVAL
    assert app(lam=None) == vb.EINVAL
    assert app(vi=None) == vb.EINVAL
    assert app(T=0) == vb.EINVAL
    assert app(T=2) == vb.EINVAL                          # pos0 + T > n_cap
    assert app(T=17, pos0=0, n_cap=64) == vb.EINVAL       # more than VECINFER_MAX_APPEND tokens
    assert app(cfg=vb.Config(128, 32, 8, 4, 3)) == vb.EUNSUPPORTED


def _decode(cfg=CFG, q=FAKE, lam=FAKE, cbk=FAKE, cbv=FAKE, ki=FAKE, vi=FAKE, sl=None, B=1, N=1024,
            n_cap=1024, S=4, variant=0, ws=None, ws_bytes=0, out=FAKE, lse=None):
    return vb.lib().vecinfer_decode_attention(C.byref(cfg.c()), q, lam, cbk, cbv, ki, vi, sl, B, N, n_cap, S,
                                              variant, ws, ws_bytes, out, lse, None)


def test_decode_argument_errors():
    assert _decode(q=None) == vb.EINVAL
    assert _decode(out=None) == vb.EINVAL
    assert _decode(B=0) == vb.EINVAL
    assert _decode(N=0) == vb.EINVAL
    assert _decode(N=2048, n_cap=1024) == vb.EINVAL
    assert _decode(S=-1) == vb.EINVAL
    assert _decode(S=vb.MAX_SPLITS + 1) == vb.EINVAL
    assert _decode(variant=7) == vb.EINVAL
    assert _decode(ki=FAKE + 1) == vb.EINVAL
    assert _decode(cfg=vb.Config(128, 32, 8, 4, 4, v_bits=4)) == vb.EUNSUPPORTED
    # valid arguments but no / too small / misaligned workspace: refused before any launch
    need = vb.vecinfer_decode_workspace_bytes(CFG, 1, 1024, 4)
    assert need > 0
    assert _decode(ws=None, ws_bytes=need) == vb.EWORKSPACE
    assert _decode(ws=FAKE, ws_bytes=need - 1) == vb.EWORKSPACE
    assert _decode(ws=FAKE + 64, ws_bytes=need) == vb.EWORKSPACE
    # no packed rows of 10 bytes: d = 8 with 10-bit codes at head dim 64
    assert _decode(cfg=vb.Config(64, 8, 1, 8, 8, 10, 10), variant=vb.VARIANT_MFMA, ws=FAKE, ws_bytes=1 << 30) == vb.EUNSUPPORTED
    # the score / value wavefront kernel: D = 128, G <= 4, d in {2, 4}, 8-bit codes
    for bad in (vb.Config(64, 8, 2, 4, 4), vb.Config(128, 16, 2, 4, 4), vb.Config(128, 8, 2, 8, 4),
                vb.Config(128, 8, 2, 4, 4, 12, 8)):
        assert _decode(cfg=bad, variant=vb.VARIANT_ROLES, ws=FAKE, ws_bytes=1 << 30) == vb.EUNSUPPORTED
    assert _decode(variant=4) == vb.EINVAL
    # more KV heads (or sequences) than a grid dimension holds
    assert _decode(cfg=vb.Config(128, 70000, 70000, 4, 4), ws=FAKE, ws_bytes=1 << 40) == vb.EUNSUPPORTED
    assert _decode(B=70000, ws=FAKE, ws_bytes=1 << 40) == vb.EUNSUPPORTED


def test_decode_residual_argument_errors():
    def res(cfg=CFG, ki=FAKE, vi=FAKE, N=1024, n_cap=1024, kr=FAKE, vr=FAKE, rl=None, R=128, r_cap=128, S=4,
            ws=None, ws_bytes=0):
        return vb.lib().vecinfer_decode_attention_residual(
            C.byref(cfg.c()), FAKE, FAKE, FAKE, FAKE, ki, vi, None, 1, N, n_cap, kr, vr, rl, R, r_cap, S, 0, ws,
            ws_bytes, FAKE, None, None)
    assert res(kr=None) == vb.EINVAL
    assert res(vr=None) == vb.EINVAL
    assert res(R=-1) == vb.EINVAL
    assert res(R=64, r_cap=32) == vb.EINVAL                     # more rows than the window holds
    assert res(N=0, R=0) == vb.EINVAL                           # nothing to attend to
    assert res(kr=FAKE + 2) == vb.EINVAL
    assert res(R=vb.MAX_RESIDUAL + 1, r_cap=256) == vb.EUNSUPPORTED
    assert res(N=0, ki=None, vi=None, R=8) == vb.EWORKSPACE     # valid without a code cache; no workspace given
    assert res(N=1024, ki=None) == vb.EINVAL                    # but codes are needed when N > 0
    need = vb.vecinfer_decode_workspace_bytes(CFG, 1, 1024, 4)
    assert res(ws=FAKE, ws_bytes=need - 1) == vb.EWORKSPACE
    assert vb.vecinfer_decode_workspace_bytes(CFG, 1, 0, 0) == vb.vecinfer_decode_workspace_bytes(CFG, 1, 1, 1) > 0


def test_decode_step_argument_errors():
    def step(cfg=CFG, kn=FAKE, vn=FAKE, ki=FAKE, vi=FAKE, N=1024, n_cap=1024, S=4, variant=0, ws=None, ws_bytes=0):
        return vb.lib().vecinfer_decode_step(C.byref(cfg.c()), FAKE, kn, vn, FAKE, FAKE, FAKE, ki, vi, None, 1, N,
                                             n_cap, S, variant, ws, ws_bytes, FAKE, None, None)
    assert step(kn=None) == vb.EINVAL
    assert step(vn=None) == vb.EINVAL
    assert step(ki=None) == vb.EINVAL
    assert step(kn=FAKE + 4) == vb.EINVAL
    assert step(N=0) == vb.EINVAL                               # the new token itself makes N >= 1
    assert step(N=2048) == vb.EINVAL
    assert step(cfg=vb.Config(128, 32, 8, 4, 4, k_bits=4)) == vb.EUNSUPPORTED
    assert step(cfg=vb.Config(64, 8, 8, 4, 8, 8, 10), variant=vb.VARIANT_MFMA, ws=FAKE, ws_bytes=1 << 30) == vb.EUNSUPPORTED
    need = vb.vecinfer_decode_workspace_bytes(CFG, 1, 1024, 4)
    assert step(ws=FAKE, ws_bytes=need - 1) == vb.EWORKSPACE


def test_kmeans_argument_errors():
    def km(cfg=CFG, x=FAKE, lam=FAKE, cbi=FAKE, cbo=FAKE, codes=FAKE, B=1, T=64, ws=FAKE, ws_bytes=1 << 30):
        return vb.lib().vecinfer_kmeans_step(C.byref(cfg.c()), x, lam, cbi, cbo, codes, None, B, T, ws, ws_bytes, None)
    assert km(x=None) == vb.EINVAL
    assert km(cbo=None) == vb.EINVAL
    assert km(codes=None) == vb.EINVAL
    assert km(T=0) == vb.EINVAL
    assert km(cfg=vb.Config(128, 32, 8, 3, 4)) == vb.EUNSUPPORTED
    need = vb.vecinfer_kmeans_workspace_bytes(CFG, True)
    assert need >= 8 * 32 * 256 * (4 * 4 + 4)
    assert km(ws=None) == vb.EWORKSPACE
    assert km(ws_bytes=need - 1) == vb.EWORKSPACE
    # the sums take the same room for every d (H_kv x D x 256 floats); the counts scale with M
    mixed = vb.Config(128, 32, 8, 2, 8)
    assert vb.vecinfer_kmeans_workspace_bytes(mixed, True) > vb.vecinfer_kmeans_workspace_bytes(mixed, False)
    assert vb.vecinfer_kmeans_workspace_bytes(vb.Config(96, 32, 8, 4, 4), True) == 0


def test_read_probe_argument_errors():
    probe = lambda src=FAKE, n=1 << 20, sink=FAKE: vb.lib().vecinfer_read_probe(src, n, sink, None)
    assert probe(src=None) == vb.EINVAL
    assert probe(sink=None) == vb.EINVAL
    assert probe(n=8) == vb.EINVAL
    assert probe(src=FAKE + 4) == vb.EINVAL


def test_calibrate_lambda_argument_errors():
    def cal(cfg=CFG, k=FAKE, lam=FAKE, B=1, T=64):
        return vb.lib().vecinfer_calibrate_lambda(C.byref(cfg.c()), k, lam, B, T, None)
    assert cal(k=None) == vb.EINVAL
    assert cal(lam=None) == vb.EINVAL
    assert cal(B=0) == vb.EINVAL
    assert cal(T=0) == vb.EINVAL
    assert cal(k=FAKE + 2) == vb.EINVAL
    assert cal(cfg=vb.Config(96, 32, 8, 4, 4)) == vb.EUNSUPPORTED


def test_wide_code_sizes_and_argument_errors():
    """10- and 12-bit codes: row bytes M b / 8 and one 2^b-entry codebook per KV head (Sec. 2.2)."""
    d8b12 = vb.Config(128, 32, 8, 8, 8, 12, 12)
    assert vb.vecinfer_index_row_bytes(d8b12, True) == 24 == d8b12.row_bytes(True)
    assert vb.vecinfer_codebook_elems(d8b12, False) == 8 * 4096 * 8 == int(np.prod(d8b12.cb_shape(False)))
    mixed = vb.Config(128, 32, 8, 4, 8, 10, 8)                       # K-d4b10 / V-d8b8
    assert vb.vecinfer_index_row_bytes(mixed, True) == 40 and vb.vecinfer_index_row_bytes(mixed, False) == 16
    assert vb.vecinfer_codebook_elems(mixed, True) == 8 * 1024 * 4
    assert vb.vecinfer_codebook_elems(mixed, False) == 8 * 16 * 256 * 8 == int(np.prod(mixed.cb_shape(False)))
    assert vb.vecinfer_index_row_bytes(CFG, True) == 32 and vb.vecinfer_codebook_elems(CFG, True) == 8 * 32 * 256 * 4
    assert vb.vecinfer_index_row_bytes(vb.Config(128, 32, 8, 2, 4, k_bits=12), True) == 0     # d = 2 has no wide form
    assert vb.vecinfer_decode_workspace_bytes(d8b12, 1, 196608, 32) == vb.vecinfer_decode_workspace_bytes(
        vb.Config(128, 32, 8, 8, 8), 1, 196608, 32)
    # the lookup-table variant reads one byte per code
    assert _decode(cfg=d8b12, variant=vb.VARIANT_LUT, ws=FAKE, ws_bytes=1 << 30) == vb.EUNSUPPORTED
    # wide codes on one side need d = 4 or 8 on the other side too
    assert _decode(cfg=vb.Config(128, 32, 8, 8, 2, 12, 8), ws=FAKE, ws_bytes=1 << 30) == vb.EUNSUPPORTED
    # the training step: fp32 sums and int32 counts for the head's one table
    assert vb.vecinfer_kmeans_workspace_bytes(d8b12, True) == 8 * 4096 * (8 * 4 + 4) + 256   # sums, counts, training state
    assert vb.lib().vecinfer_kmeans_step(C.byref(d8b12.c()), FAKE, FAKE, FAKE, FAKE, FAKE, None, 1, 64, FAKE, 1024,
                                         None) == vb.EWORKSPACE
    assert _enc_keys(cfg=d8b12, k=None) == vb.EINVAL


def test_workspace_size_and_auto_splits():
    assert vb.vecinfer_decode_workspace_bytes(vb.Config(96, 32, 8, 4, 4), 1, 1024, 4) == 0
    assert vb.vecinfer_decode_workspace_bytes(CFG, 1, 1024, vb.MAX_SPLITS + 1) == 0
    a = vb.vecinfer_decode_workspace_bytes(CFG, 1, 196608, 32)
    # partial outputs dominate: B * Hq * S * D floats, plus (m, l)
    assert a >= 1 * 32 * 32 * 128 * 4 and a % 256 == 0
    assert vb.vecinfer_decode_workspace_bytes(CFG, 2, 196608, 32) > a
    s = vb.vecinfer_decode_auto_splits(CFG, 1, 196608)
    assert 1 <= s <= vb.MAX_SPLITS
    assert vb.vecinfer_decode_auto_splits(CFG, 32, 8192) >= 1
    assert vb.vecinfer_decode_auto_splits(CFG, 1, 100) == 1        # short sequences are not split
    assert vb.vecinfer_decode_auto_splits(CFG, 0, 100) == vb.EINVAL
    assert vb.vecinfer_decode_workspace_bytes(CFG, 1, 196608, 0) == vb.vecinfer_decode_workspace_bytes(CFG, 1, 196608, s)


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(TypeError):
        vb.vecinfer_encode_values(CFG, torch.zeros(1, 8, 4, 128, dtype=torch.float16),
                                  torch.zeros(8, 32, 256, 4, dtype=torch.float16),
                                  torch.zeros(1, 8, 8, 32, dtype=torch.uint8))


def test_tiled_value_codes_argument_errors():
    tiled = vb.Config(128, 32, 8, 4, 4, v_tiled=1)
    # tiled value codes are one byte per code
    assert _decode(cfg=vb.Config(128, 32, 8, 8, 8, 12, 12, 1), ws=FAKE, ws_bytes=1 << 30) == vb.EUNSUPPORTED
    assert _decode(cfg=vb.Config(128, 32, 8, 4, 4, v_tiled=2), ws=FAKE, ws_bytes=1 << 30) == vb.EUNSUPPORTED
    # .. and need the 16 value sub-spaces the block order is made of
    assert _decode(cfg=vb.Config(64, 8, 8, 4, 8, v_tiled=1), ws=FAKE, ws_bytes=1 << 30) == vb.EUNSUPPORTED
    assert _enc_vals(cfg=vb.Config(64, 8, 8, 4, 8, v_tiled=1), T=64, n_cap=64) == vb.EUNSUPPORTED
    # whole 64-token blocks
    assert _decode(cfg=tiled, N=1000, n_cap=1000, ws=FAKE, ws_bytes=1 << 30) == vb.EINVAL
    assert _enc_vals(cfg=tiled, T=4, n_cap=100) == vb.EINVAL
    # the lookup-table variant reads rows
    assert _decode(cfg=tiled, variant=vb.VARIANT_LUT, ws=FAKE, ws_bytes=1 << 30) == vb.EUNSUPPORTED
    # export
    exp = lambda cfg=tiled, src=FAKE, dst=FAKE + 4096, B=1, N=64, n_cap=64: vb.lib().vecinfer_export_value_codes(
        C.byref(cfg.c()), src, dst, B, N, n_cap, None)
    assert exp(src=None) == vb.EINVAL
    assert exp(dst=FAKE) == vb.EINVAL                       # in place
    assert exp(N=0) == vb.EINVAL
    assert exp(N=65) == vb.EINVAL
    assert exp(N=60, n_cap=100) == vb.EINVAL
    assert exp(cfg=vb.Config(128, 32, 8, 8, 8, 8, 12)) == vb.EUNSUPPORTED


def test_tiled_layout_formula():
    """The test-side tiling (written from the header's formula) is a permutation of each 64-token
    block, and a lane finds its 16 R bytes as 16 from each of the block's R slabs of 1 KB: the bytes
    the header promises."""
    from helpers import tile_value_codes
    for M in (16, 32, 64):
        R = M // 16
        rows = np.arange(2 * 128 * M, dtype=np.int64).reshape(1, 2, 128, M)
        tiled = tile_value_codes(rows).reshape(1, 2, 128 * M)
        for h in range(2):
            for blk in range(2):
                got = np.sort(tiled[0, h, blk * 64 * M:(blk + 1) * 64 * M])
                np.testing.assert_array_equal(got, np.sort(rows[0, h, blk * 64:(blk + 1) * 64].reshape(-1)))
        # lane (kg, col) of block 1: tokens 64 + 16 st + 4 v + kg, sub-spaces R col .. R col + R - 1
        kg, col = 2, 5
        lane = kg * 16 + col
        run = np.concatenate([tiled[0, 1, 64 * M + s * 1024 + lane * 16: 64 * M + s * 1024 + lane * 16 + 16]
                              for s in range(R)])
        want = [rows[0, 1, 64 + 16 * st + 4 * v + kg, R * col + r] for st in range(4) for v in range(4) for r in range(R)]
        np.testing.assert_array_equal(run, np.array(want))


def test_static_entry_refuses_before_any_device_call():
    """vecinfer_decode_attention_static: argument and size checks come before the device is
    touched, so they can be exercised on the host."""
    def call(cfg=CFG, B=1, N=1024, splits=4, q=FAKE):
        return vb.lib().vecinfer_decode_attention_static(C.byref(cfg.c()), q, FAKE, FAKE, FAKE, FAKE, FAKE, None,
                                                         B, N, N, splits, vb.VARIANT_AUTO, FAKE, None, None)
    assert vb.lib().vecinfer_decode_attention_static(None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 1, 64, 64, 1,
                                                     vb.VARIANT_AUTO, FAKE, None, None) == vb.EINVAL
    assert call(cfg=vb.Config(96, 32, 8, 4, 4)) == vb.EUNSUPPORTED
    assert call(B=0) == vb.EINVAL
    assert call(N=0) == vb.EINVAL
    assert call(splits=vb.MAX_SPLITS + 1) == vb.EINVAL
    # 8 sequences x 32 heads x 64 splits x 130 floats = 8.5 MB of partials: over the 4 MiB array
    assert vb.vecinfer_decode_workspace_bytes(CFG, 8, 4096, 64) > vb.STATIC_SCRATCH_BYTES
    assert call(B=8, N=4096, splits=64) == vb.EWORKSPACE
    # the headline shape fits with room to spare
    assert vb.vecinfer_decode_workspace_bytes(CFG, 1, 196608, 32) < vb.STATIC_SCRATCH_BYTES // 4
