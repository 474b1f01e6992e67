"""GPU parity: the HIP path (through the C ABI) against the float64 oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_06175_amd import binding as vb
from paper_2510_06175_amd import synth

from helpers import (assert_decode_close, assert_indices_match, cfg_of, dev, gpu_decode, gpu_encode)

pytestmark = pytest.mark.gpu

VARIANTS = {"lut": vb.VARIANT_LUT, "mfma": vb.VARIANT_MFMA}


def _supported(shape, variant):
    return variant == vb.VARIANT_LUT or (shape.D == 128 and shape.G == 4 and shape.d_k in (2, 4)
                                         and shape.d_v == shape.d_k)


# ------------------------------------------------------------------ decode, small shapes

SMALL = [
    # B, Hq, Hkv, D, N, d_k, d_v   (several tiles plus a ragged tail; every supported family)
    synth.Shape(1, 1, 1, 128, 1000, 4, 4),
    synth.Shape(2, 8, 2, 128, 777, 4, 4),
    synth.Shape(2, 8, 2, 128, 1500, 2, 2),
    synth.Shape(1, 4, 2, 64, 513, 4, 2),
    synth.Shape(1, 8, 1, 64, 300, 8, 8),
    synth.Shape(3, 4, 4, 128, 65, 2, 8),
    synth.Shape(1, 4, 1, 128, 4099, 4, 4),
]


@pytest.mark.parametrize("vname", list(VARIANTS))
@pytest.mark.parametrize("shape", SMALL, ids=lambda s: f"B{s.B}h{s.Hq}-{s.Hkv}D{s.D}N{s.N}k{s.d_k}v{s.d_v}")
@pytest.mark.parametrize("splits", [1, 3, 0])
def test_decode_small(shape, splits, vname):
    variant = VARIANTS[vname]
    if not _supported(shape, variant):
        pytest.skip("variant does not cover this configuration")
    x = synth.decode_inputs(shape, seed=shape.N + splits)
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    got = gpu_decode(shape, x, num_splits=splits, variant=variant)
    assert_decode_close(*got, *ref, what=f"{vname} splits={splits}")


@pytest.mark.parametrize("vname", list(VARIANTS))
def test_decode_ragged_batch_and_degenerate_lengths(vname):
    """seq_lens ragged, one sequence of a single token, one of length 0 (o = 0, L = -inf),
    N below the cache capacity."""
    shape = synth.Shape(4, 8, 2, 128, 900, 4, 4)
    variant = VARIANTS[vname]
    x = synth.decode_inputs(shape, seed=5, n_cap=1024)
    lens = np.array([900, 1, 0, 333])
    got_o, got_l = gpu_decode(shape, x, seq_lens=lens, N=900, num_splits=4, variant=variant)
    keep = [0, 1, 3]
    sub = {k: (v[keep] if k in ("q", "k_idx", "v_idx") else v) for k, v in x.items()}
    ref_o, ref_l = oracle.decode_attention(sub["q"], sub["lam"], sub["cb_k"], sub["cb_v"], sub["k_idx"],
                                           sub["v_idx"], lens[keep])
    assert_decode_close(got_o[keep], got_l[keep], ref_o, ref_l, what=vname)
    assert (got_o[2] == 0).all() and np.isneginf(got_l[2]).all()


@pytest.mark.parametrize("vname", list(VARIANTS))
def test_decode_split_count_invariance_and_determinism(vname):
    shape = synth.Shape(1, 8, 2, 128, 6000, 4, 4)
    variant = VARIANTS[vname]
    x = synth.decode_inputs(shape, seed=9)
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    outs = {}
    for S in (1, 2, 32, 64, 256):
        outs[S] = gpu_decode(shape, x, num_splits=S, variant=variant)
        assert_decode_close(*outs[S], *ref, what=f"{vname} S={S}")
    again = gpu_decode(shape, x, num_splits=32, variant=variant)
    np.testing.assert_array_equal(again[0], outs[32][0])
    np.testing.assert_array_equal(again[1], outs[32][1])


@pytest.mark.parametrize("vname", list(VARIANTS))
def test_decode_workspace_reuse_across_calls(vname):
    """One workspace (never initialised) serves successive calls with different split counts."""
    shape = synth.Shape(2, 8, 2, 128, 3000, 4, 4)
    variant = VARIANTS[vname]
    x = synth.decode_inputs(shape, seed=10)
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    ws = vb.new_workspace(cfg_of(shape), shape.B, shape.N, 16)
    for S in (16, 5, 16, 1):
        got = gpu_decode(shape, x, num_splits=S, variant=variant, ws=ws)
        assert_decode_close(*got, *ref, what=f"{vname} reuse S={S}")


@pytest.mark.parametrize("vname", list(VARIANTS))
def test_decode_peaked_attention(vname):
    """A query aligned with one token's dequantized key: softmax is nearly one-hot and the
    output must be that token's dequantized value (degenerate, precision-critical case)."""
    shape = synth.Shape(1, 4, 1, 128, 2048, 4, 4)
    variant = VARIANTS[vname]
    x = synth.decode_inputs(shape, seed=12)
    x["lam"][:] = 1.0
    H = oracle.hadamard(128)
    for h, tok in enumerate((0, 777, 2047, 1024)):
        khat = oracle.vq_dequantize(x["k_idx"][0, 0, tok:tok + 1], x["cb_k"][0])[0]
        x["q"][0, h] = (3.0 * (khat @ H.T)).astype(np.float16)      # q~ = q H ~ 3 khat
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    got = gpu_decode(shape, x, num_splits=4, variant=variant)
    assert_decode_close(*got, *ref, what=vname)


# ------------------------------------------------------------------ encode

ENC_SHAPES = [
    synth.Shape(1, 1, 1, 128, 200, 4, 4),
    synth.Shape(2, 4, 2, 128, 129, 2, 8),
    synth.Shape(1, 2, 2, 64, 70, 4, 2),
    synth.Shape(1, 3, 3, 64, 64, 8, 8),
]


@pytest.mark.parametrize("shape", ENC_SHAPES, ids=lambda s: f"B{s.B}Hkv{s.Hkv}D{s.D}T{s.N}k{s.d_k}v{s.d_v}")
def test_encode_small(shape):
    e = synth.encode_inputs(shape, seed=shape.N, n_outlier=3)
    lam = np.stack([oracle.smoothing_factors(e["k"][:, h]) for h in range(shape.Hkv)]).astype(np.float32)
    ref_k, gap_k = oracle.encode_keys(e["k"], lam, e["cb_k"], want_gap=True)
    ref_v, gap_v = oracle.encode_values(e["v"], e["cb_v"], want_gap=True)
    got_k, got_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"])
    assert_indices_match(got_k, ref_k, gap_k, "keys")
    assert_indices_match(got_v, ref_v, gap_v, "values")


def test_encode_append_at_offset_leaves_other_rows_untouched():
    """Eq. 9: decode-time append = encode with T = 1 at pos0 = current length."""
    shape = synth.Shape(2, 4, 2, 128, 1, 4, 4)
    e = synth.encode_inputs(shape, seed=77, n_outlier=3)
    lam = synth.lognormal_lambda(synth.rng(3), 2, 128)
    got_k, got_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"], pos0=37, n_cap=50)
    ref_k = oracle.encode_keys(e["k"], lam, e["cb_k"])
    ref_v = oracle.encode_values(e["v"], e["cb_v"])
    np.testing.assert_array_equal(got_k[:, :, 37], ref_k[:, :, 0])
    np.testing.assert_array_equal(got_v[:, :, 37], ref_v[:, :, 0])
    mask = np.ones(50, bool)
    mask[37] = False
    assert (got_k[:, :, mask] == 0xEE).all() and (got_v[:, :, mask] == 0xEE).all()


def test_encode_short_and_tiled_kernels_agree():
    """Short inputs (decode-time append) take a per-token kernel, long ones a tiled kernel:
    same butterfly order and distance arithmetic, so identical codes on identical tokens."""
    shape = synth.Shape(2, 8, 2, 128, 40, 4, 2)
    e = synth.encode_inputs(shape, seed=41, n_outlier=3)
    lam = synth.lognormal_lambda(synth.rng(4), 2, 128)
    long_k, long_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"])
    short_k, short_v = gpu_encode(shape, k=e["k"][:, :, :9], lam=lam, cb_k=e["cb_k"], v=e["v"][:, :, :9],
                                  cb_v=e["cb_v"])
    np.testing.assert_array_equal(short_k, long_k[:, :, :9])
    np.testing.assert_array_equal(short_v, long_v[:, :, :9])
    ref_k, gap = oracle.encode_keys(e["k"][:, :, :9], lam, e["cb_k"], want_gap=True)
    assert_indices_match(short_k, ref_k, gap, "short keys")


def test_append_kv_equals_separate_encodes():
    """vecinfer_append_kv (one launch) writes exactly the codes of encode_keys + encode_values,
    for mixed sub-vector dims, at an offset, leaving the other rows alone."""
    shape = synth.Shape(2, 8, 2, 128, 3, 4, 2)
    e = synth.encode_inputs(shape, seed=43, n_outlier=3)
    lam = synth.lognormal_lambda(synth.rng(6), 2, 128)
    sep_k, sep_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"], pos0=5, n_cap=16)
    cfg = cfg_of(shape)
    k_idx = torch.full((2, 2, 16, shape.Mk), 0xEE, dtype=torch.uint8, device="cuda")
    v_idx = torch.full((2, 2, 16, shape.Mv), 0xEE, dtype=torch.uint8, device="cuda")
    vb.vecinfer_append_kv(cfg, dev(e["k"]), dev(e["v"]), dev(lam), dev(e["cb_k"]), dev(e["cb_v"]), k_idx, v_idx, pos0=5)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(k_idx.cpu().numpy(), sep_k)
    np.testing.assert_array_equal(v_idx.cpu().numpy(), sep_v)
    ref_k, gap = oracle.encode_keys(e["k"], lam, e["cb_k"], want_gap=True)
    assert_indices_match(sep_k[:, :, 5:8], ref_k, gap, "append keys")


def test_encode_planted_codes_and_ties():
    """Rows built from centroids come back as exactly those codes; duplicate centroids resolve
    to the lower index."""
    shape = synth.Shape(1, 2, 2, 128, 96, 4, 4)
    g = synth.rng(31)
    cb = synth.codebooks(g, 2, 32, 4)
    cb[:, :, 200] = cb[:, :, 17]
    want = g.integers(0, 256, size=(1, 2, 96, 32), dtype=np.uint8)
    V = np.stack([[oracle.vq_dequantize(want[0, h], cb[h]) for h in range(2)]]).astype(np.float16)
    (got_v,) = gpu_encode(shape, v=V, cb_v=cb)
    expect = np.where(want == 200, 17, want)
    np.testing.assert_array_equal(got_v, expect)


# ------------------------------------------------------------------ the BASELINE configurations

def test_config1_tiny_encode_then_decode():
    """Config 1: 1 head, N 4096, keys with 4 outlier channels x20, lambda by Eq. 4, b2d4."""
    shape = synth.TINY
    e = synth.encode_inputs(shape, seed=1, n_outlier=4)
    lam = oracle.smoothing_factors(e["k"][0, 0])[None, :].astype(np.float32)
    ref_k, gap_k = oracle.encode_keys(e["k"], lam, e["cb_k"], want_gap=True)
    ref_v, gap_v = oracle.encode_values(e["v"], e["cb_v"], want_gap=True)
    got_k, got_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"])
    assert_indices_match(got_k, ref_k, gap_k, "config1 keys")
    assert_indices_match(got_v, ref_v, gap_v, "config1 values")
    x = {"q": e["q"], "lam": lam, "cb_k": e["cb_k"], "cb_v": e["cb_v"], "k_idx": got_k, "v_idx": got_v}
    ref = oracle.decode_attention(e["q"], lam, e["cb_k"], e["cb_v"], got_k, got_v)
    for vname, variant in VARIANTS.items():
        if _supported(shape, variant):
            assert_decode_close(*gpu_decode(shape, x, variant=variant), *ref, what=f"config1 {vname}")


@pytest.mark.parametrize("name,shape", [("config2-32k", synth.LLAMA8B_32K), ("config3-batch32", synth.LLAMA8B_BATCH32),
                                        ("config4-196k-b2d4", synth.LLAMA8B_196K),
                                        ("config4-196k-b4d2", synth.LLAMA8B_196K_B4D2)])
def test_decode_full_size_configs(name, shape):
    """Configs 2-4 at full size, in the launch configuration the benchmark times (auto variant,
    auto splits), every output element against the oracle."""
    x = synth.decode_inputs(shape, seed={"config2-32k": 2, "config3-batch32": 3}.get(name, 4))
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    got = gpu_decode(shape, x)
    worst = assert_decode_close(*got, *ref, what=name)
    print(f"[{name}] worst max|err|/||out||inf = {worst:.2e}")
    if shape.N >= 100000:                       # the split sweep of config 4
        for S in (16, 64, 256):
            assert_decode_close(*gpu_decode(shape, x, num_splits=S), *ref, what=f"{name} S={S}")


def test_config5_cache_fill_then_decode():
    """Config 5: encode 65536 tokens x 8 KV heads (keys with 3 outlier channels x20, lambda by
    Eq. 4), indices bit-exact up to logged near-ties, then one decode step over the fresh cache."""
    shape = synth.ENCODE_64K
    e = synth.encode_inputs(shape, seed=5, n_outlier=3)
    lam = np.stack([oracle.smoothing_factors(e["k"][:, h]) for h in range(shape.Hkv)]).astype(np.float32)
    got_k, got_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"])
    ref_k, gap_k = oracle.encode_keys(e["k"], lam, e["cb_k"], want_gap=True)
    assert_indices_match(got_k, ref_k, gap_k, "config5 keys")
    del ref_k, gap_k
    ref_v, gap_v = oracle.encode_values(e["v"], e["cb_v"], want_gap=True)
    assert_indices_match(got_v, ref_v, gap_v, "config5 values")
    del ref_v, gap_v
    x = {"q": e["q"], "lam": lam, "cb_k": e["cb_k"], "cb_v": e["cb_v"], "k_idx": got_k, "v_idx": got_v}
    ref = oracle.decode_attention(e["q"], lam, e["cb_k"], e["cb_v"], got_k, got_v)
    assert_decode_close(*gpu_decode(shape, x), *ref, what="config5 decode")
