"""GPU parity for the tiled layout of the value code cache (cfg.v_tiled = 1): the same N x M code
matrix stored in blocks of 64 tokens in the order the matrix-core kernel's lanes consume it.
Through the C ABI: against the float64 oracle, and bit for bit against the rows layout (the two
layouts feed the same arithmetic in the same order)."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_2510_06175_amd import binding as vb
from paper_2510_06175_amd import synth

from helpers import assert_decode_close, assert_indices_match, cfg_of, dev, gpu_decode, gpu_encode, tile_value_codes

pytestmark = pytest.mark.gpu


def _id(s):
    return f"B{s.B}h{s.Hq}-{s.Hkv}D{s.D}N{s.N}k{s.d_k}v{s.d_v}"


def _cap(n):
    return (n + 63) // 64 * 64


def _export(shape, v_tiled_dev, N=None):
    rows = torch.full_like(v_tiled_dev, 0xAB)
    vb.vecinfer_export_value_codes(cfg_of(shape, 1), v_tiled_dev, rows, N=N)
    torch.cuda.synchronize()
    return rows.cpu().numpy()


# every (d_k, d_v) pair of 8-bit codes the matrix-core kernel covers, both head dims, G = 4, 1, 8, 3,
# lengths with several tiles per wavefront and a ragged tail
SHAPES = [
    synth.Shape(2, 8, 2, 128, 777, 4, 4),
    synth.Shape(1, 8, 2, 128, 4099, 4, 4),
    synth.Shape(1, 2, 2, 128, 1300, 2, 2),
    synth.Shape(1, 16, 2, 128, 600, 2, 4),
    synth.Shape(2, 8, 2, 128, 900, 4, 2),
    synth.Shape(1, 3, 1, 128, 1000, 8, 8),
    synth.Shape(1, 8, 2, 128, 700, 8, 4),
    synth.Shape(1, 8, 2, 128, 650, 8, 2),
    synth.Shape(2, 8, 2, 128, 800, 4, 8),
    synth.Shape(1, 8, 2, 128, 500, 2, 8),
    synth.Shape(2, 8, 2, 64, 777, 4, 4),
    synth.Shape(1, 8, 2, 64, 1500, 8, 4),
    synth.Shape(1, 4, 1, 64, 900, 8, 2),
    synth.Shape(1, 16, 2, 64, 640, 2, 2),
    synth.Shape(1, 8, 2, 64, 333, 2, 4),
    synth.Shape(1, 8, 2, 64, 1100, 4, 2),
]


@pytest.mark.parametrize("shape", SHAPES, ids=_id)
@pytest.mark.parametrize("splits", [1, 3, 0])
def test_decode_tiled(shape, splits):
    x = synth.decode_inputs(shape, seed=shape.N + splits, n_cap=_cap(shape.N))
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"][:, :, :shape.N],
                                  x["v_idx"][:, :, :shape.N])
    rows = gpu_decode(shape, x, N=shape.N, num_splits=splits)
    got = gpu_decode(shape, dict(x, v_idx=tile_value_codes(x["v_idx"])), N=shape.N, num_splits=splits, v_tiled=1)
    assert_decode_close(*got, *ref, what=f"tiled {_id(shape)} S={splits}")
    np.testing.assert_array_equal(got[0], rows[0])
    np.testing.assert_array_equal(got[1], rows[1])


@pytest.mark.parametrize("shape", [synth.Shape(2, 8, 2, 128, 777, 4, 4), synth.Shape(1, 4, 1, 128, 4099, 2, 2),
                                   synth.Shape(1, 6, 2, 128, 1500, 4, 2), synth.Shape(2, 4, 2, 128, 900, 2, 4)], ids=_id)
@pytest.mark.parametrize("splits", [1, 3, 0])
def test_decode_tiled_roles_variant(shape, splits):
    """The score / value wavefront kernel reads the tiled value codes too: bit-identical to its own
    result on rows, and within the bar of the oracle."""
    x = synth.decode_inputs(shape, seed=shape.N + splits + 100, n_cap=_cap(shape.N))
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"][:, :, :shape.N],
                                  x["v_idx"][:, :, :shape.N])
    rows = gpu_decode(shape, x, N=shape.N, num_splits=splits, variant=vb.VARIANT_ROLES)
    got = gpu_decode(shape, dict(x, v_idx=tile_value_codes(x["v_idx"])), N=shape.N, num_splits=splits, v_tiled=1,
                     variant=vb.VARIANT_ROLES)
    assert_decode_close(*got, *ref, what=f"tiled roles {_id(shape)} S={splits}")
    np.testing.assert_array_equal(got[0], rows[0])
    np.testing.assert_array_equal(got[1], rows[1])


def test_decode_tiled_ragged_and_degenerate_lengths():
    shape = synth.Shape(4, 8, 2, 128, 900, 4, 4)
    x = synth.decode_inputs(shape, seed=5, n_cap=1024)
    lens = np.array([900, 1, 0, 333])
    got = gpu_decode(shape, dict(x, v_idx=tile_value_codes(x["v_idx"])), seq_lens=lens, N=900, num_splits=4, v_tiled=1)
    keep = [0, 1, 3]                                    # the oracle takes no empty sequence
    ref = oracle.decode_attention(x["q"][keep], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"][keep], x["v_idx"][keep],
                                  lens[keep])
    assert_decode_close(got[0][keep], got[1][keep], *ref, what="tiled ragged")
    assert (got[0][2] == 0).all() and np.isneginf(got[1][2]).all()


def test_decode_tiled_full_size_196k_equals_rows():
    shape = synth.LLAMA8B_196K
    x = synth.decode_inputs(shape, seed=4)
    rows = gpu_decode(shape, x)
    got = gpu_decode(shape, dict(x, v_idx=tile_value_codes(x["v_idx"])), v_tiled=1)
    np.testing.assert_array_equal(got[0], rows[0])
    np.testing.assert_array_equal(got[1], rows[1])


# ------------------------------------------------------------------ cache fill

@pytest.mark.parametrize("shape,pos0", [
    (synth.Shape(2, 4, 2, 128, 300, 4, 4), 0),          # tiled kernel, ragged last tile
    (synth.Shape(1, 2, 2, 128, 200, 4, 2), 37),         # written from the middle of a block
    (synth.Shape(1, 2, 2, 128, 130, 4, 8), 64),
    (synth.Shape(2, 2, 2, 64, 257, 4, 4), 5),
    (synth.Shape(1, 2, 2, 128, 7, 4, 4), 61),           # per-token kernel, across a block boundary
    (synth.Shape(1, 2, 1, 64, 3, 8, 2), 0),
], ids=lambda v: _id(v) if isinstance(v, synth.Shape) else f"pos{v}")
def test_encode_values_tiled(shape, pos0):
    e = synth.encode_inputs(shape, seed=shape.N + pos0, n_outlier=3)
    cap = _cap(pos0 + shape.N + 10)
    (rows,) = gpu_encode(shape, v=e["v"], cb_v=e["cb_v"], pos0=pos0, n_cap=cap)
    (tiled,) = gpu_encode(shape, v=e["v"], cb_v=e["cb_v"], pos0=pos0, n_cap=cap, v_tiled=1)
    # the same bytes, each at its place in the tiled layout; nothing else is touched (0xEE fill)
    np.testing.assert_array_equal(tiled, tile_value_codes(rows))
    # and back to rows through the library
    back = _export(shape, dev(tiled), N=pos0 + shape.N)
    np.testing.assert_array_equal(back[:, :, :pos0 + shape.N], rows[:, :, :pos0 + shape.N])
    assert (back[:, :, pos0 + shape.N:] == 0xAB).all()
    # against the oracle
    ref, gap = oracle.encode_values(e["v"], e["cb_v"], want_gap=True)
    assert_indices_match(rows[:, :, pos0:pos0 + shape.N], ref, gap, what="values")


def test_append_kv_tiled():
    shape = synth.Shape(2, 8, 2, 128, 200, 4, 4)
    cfg_r, cfg_t = cfg_of(shape), cfg_of(shape, 1)
    x = synth.decode_inputs(shape, seed=9, n_cap=256)
    g = synth.rng(10)
    T = 5
    k_new = synth.values(g, shape.B, shape.Hkv, T, shape.D)
    v_new = synth.values(g, shape.B, shape.Hkv, T, shape.D)
    out = []
    for cfg, v0 in ((cfg_r, x["v_idx"]), (cfg_t, tile_value_codes(x["v_idx"]))):
        k_idx, v_idx = dev(x["k_idx"]), dev(v0)
        vb.vecinfer_append_kv(cfg, dev(k_new), dev(v_new), dev(x["lam"]), dev(x["cb_k"]), dev(x["cb_v"]), k_idx, v_idx,
                              pos0=shape.N - 2)
        torch.cuda.synchronize()
        out.append((k_idx.cpu().numpy(), v_idx.cpu().numpy()))
    np.testing.assert_array_equal(out[0][0], out[1][0])
    np.testing.assert_array_equal(tile_value_codes(out[0][1]), out[1][1])


# ------------------------------------------------------------------ the whole step

def _step(shape, x, k_new, v_new, v_tiled, seq_lens=None, N=None, num_splits=0):
    cfg = cfg_of(shape, v_tiled)
    k_idx = dev(x["k_idx"])
    v_idx = dev(tile_value_codes(x["v_idx"]) if v_tiled else x["v_idx"])
    B, n_cap = k_idx.shape[0], k_idx.shape[2]
    N = n_cap if N is None else N
    ws = vb.new_workspace(cfg, B, N, num_splits)
    out = torch.full((B, shape.Hq, shape.D), float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full((B, shape.Hq), float("nan"), dtype=torch.float32, device="cuda")
    sl = None if seq_lens is None else torch.as_tensor(np.asarray(seq_lens), dtype=torch.int32).cuda()
    vb.vecinfer_decode_step(cfg, dev(x["q"]), dev(k_new), dev(v_new), dev(x["lam"]), dev(x["cb_k"]), dev(x["cb_v"]),
                            k_idx, v_idx, ws, out, lse=lse, seq_lens=sl, N=N, num_splits=num_splits)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy(), k_idx.cpu().numpy(), v_idx.cpu().numpy()


@pytest.mark.parametrize("shape", [
    synth.Shape(2, 8, 2, 128, 777, 4, 4),
    synth.Shape(1, 8, 2, 128, 2049, 2, 2),
    synth.Shape(1, 16, 2, 128, 640, 8, 8),
    synth.Shape(1, 8, 2, 64, 900, 8, 4),
    synth.Shape(1, 4, 1, 128, 1000, 4, 8),
], ids=_id)
@pytest.mark.parametrize("splits", [1, 5, 0])
def test_decode_step_tiled(shape, splits):
    """The fused step on a tiled cache writes the new token's codes at their tiled places and returns
    the numbers of the step on the rows cache, bit for bit."""
    x = synth.decode_inputs(shape, seed=shape.N + 31, n_cap=_cap(shape.N))
    g = synth.rng(shape.N + 32)
    k_new = synth.values(g, shape.B, shape.Hkv, 1, shape.D)
    v_new = synth.values(g, shape.B, shape.Hkv, 1, shape.D)
    r = _step(shape, x, k_new, v_new, 0, N=shape.N, num_splits=splits)
    t = _step(shape, x, k_new, v_new, 1, N=shape.N, num_splits=splits)
    np.testing.assert_array_equal(t[0], r[0])
    np.testing.assert_array_equal(t[1], r[1])
    np.testing.assert_array_equal(t[2], r[2])
    np.testing.assert_array_equal(t[3], tile_value_codes(r[3]))
    # and against the oracle: the cache with the new token's codes at row N - 1
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], r[2][:, :, :shape.N], r[3][:, :, :shape.N])
    assert_decode_close(t[0].astype(np.float64), t[1].astype(np.float64), *ref, what=f"tiled step {_id(shape)}")


def test_decode_step_tiled_full_size_196k():
    """The configuration bench.py times (32 / 8 heads, 196608 tokens, b2d4, tiled value codes): the
    whole step equals the step on the rows cache bit for bit (which the parity tests check against
    the oracle at this size), and the new token's codes sit at their tiled places."""
    shape = synth.LLAMA8B_196K
    x = synth.decode_inputs(shape, seed=4)
    g = synth.rng(45)
    k_new = synth.values(g, shape.B, shape.Hkv, 1, shape.D)
    v_new = synth.values(g, shape.B, shape.Hkv, 1, shape.D)
    r = _step(shape, x, k_new, v_new, 0)
    t = _step(shape, x, k_new, v_new, 1)
    np.testing.assert_array_equal(t[0], r[0])
    np.testing.assert_array_equal(t[1], r[1])
    np.testing.assert_array_equal(t[2], r[2])
    np.testing.assert_array_equal(t[3], tile_value_codes(r[3]))


def test_decode_step_tiled_ragged():
    shape = synth.Shape(4, 8, 2, 128, 900, 4, 4)
    x = synth.decode_inputs(shape, seed=41, n_cap=1024)
    g = synth.rng(42)
    k_new = synth.values(g, shape.B, shape.Hkv, 1, shape.D)
    v_new = synth.values(g, shape.B, shape.Hkv, 1, shape.D)
    lens = [900, 1, 0, 334]
    r = _step(shape, x, k_new, v_new, 0, seq_lens=lens, N=900, num_splits=4)
    t = _step(shape, x, k_new, v_new, 1, seq_lens=lens, N=900, num_splits=4)
    np.testing.assert_array_equal(t[0], r[0])
    np.testing.assert_array_equal(t[1], r[1])
    np.testing.assert_array_equal(t[3], tile_value_codes(r[3]))


def test_tiled_refusals():
    """Shapes the tiled layout does not take are refused on the host, before any launch."""
    shape = synth.Shape(1, 8, 2, 128, 100, 4, 4)
    x = synth.decode_inputs(shape, seed=1, n_cap=100)           # capacity not a multiple of 64
    with pytest.raises(vb.VecInferError) as e:
        gpu_decode(shape, x, v_tiled=1)
    assert e.value.code == vb.EINVAL
    x = synth.decode_inputs(shape, seed=1, n_cap=128)
    with pytest.raises(vb.VecInferError) as e:
        gpu_decode(shape, x, N=100, variant=vb.VARIANT_LUT, v_tiled=1)
    assert e.value.code == vb.EUNSUPPORTED
