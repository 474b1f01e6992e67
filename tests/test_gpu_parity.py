"""GPU parity: the HIP path (through the C ABI) against the float64 oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_06175_amd import binding as vb
from paper_2510_06175_amd import synth

from helpers import (assert_decode_close, assert_indices_match, cfg_of, dev, gpu_decode, gpu_decode_residual,
                     gpu_encode)

pytestmark = pytest.mark.gpu

VARIANTS = {"lut": vb.VARIANT_LUT, "mfma": vb.VARIANT_MFMA, "roles": vb.VARIANT_ROLES}


def _supported(shape, variant):
    if variant == vb.VARIANT_ROLES:       # score / value wavefront kernel: 8-bit codes, D = 128, G <= 4, d in {2, 4}
        return shape.D == 128 and shape.G <= 4 and shape.d_k in (2, 4) and shape.d_v in (2, 4)
    return variant == vb.VARIANT_LUT or (shape.D in (64, 128) and shape.G <= 8 and shape.d_k in (2, 4, 8)
                                         and shape.d_v in (2, 4, 8))


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
    synth.Shape(2, 8, 2, 64, 777, 4, 4),          # head dim 64 on the matrix-core path
    synth.Shape(1, 8, 2, 64, 1500, 2, 2),
    synth.Shape(1, 4, 1, 64, 4099, 4, 4),
    synth.Shape(2, 4, 2, 128, 777, 4, 4),         # G = 2 and G = 1 on the matrix-core path (spare head slots)
    synth.Shape(1, 3, 3, 128, 1000, 2, 2),
    synth.Shape(2, 2, 2, 64, 900, 4, 4),
    synth.Shape(2, 8, 2, 128, 777, 2, 4),         # keys and values quantized differently (Sec. 3.2)
    synth.Shape(1, 8, 2, 128, 900, 4, 2),
    synth.Shape(1, 8, 2, 64, 1100, 2, 4),
    synth.Shape(1, 16, 2, 128, 777, 4, 4),        # G = 8: two passes of four heads over the same operands
    synth.Shape(2, 8, 1, 64, 513, 2, 2),
    synth.Shape(1, 7, 1, 128, 900, 4, 4),         # G = 7, G = 3: spare head slots
    synth.Shape(1, 6, 2, 128, 600, 4, 2),
    synth.Shape(2, 8, 2, 128, 777, 8, 8),         # d = 8 (one bit per element) on the matrix-core path
    synth.Shape(1, 4, 1, 128, 1000, 4, 8),        # 2-bit keys, 1-bit values
    synth.Shape(1, 8, 2, 64, 900, 8, 4),
    synth.Shape(1, 16, 2, 128, 600, 8, 8),
    synth.Shape(1, 4, 1, 128, 500, 2, 8),
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


# ------------------------------------------------------------------ the benchmark configurations at full size

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


# ------------------------------------------------------------------ residual window (Sec. 4.1)

RESIDUAL = [
    # shape, rows in the window
    (synth.Shape(2, 8, 2, 128, 777, 4, 4), 128),
    (synth.Shape(1, 8, 2, 128, 1500, 2, 2), 37),
    (synth.Shape(1, 4, 2, 64, 513, 4, 2), 128),
    (synth.Shape(1, 8, 1, 64, 300, 8, 8), 5),
    (synth.Shape(3, 4, 4, 128, 65, 2, 8), 1),
    (synth.Shape(2, 8, 2, 64, 777, 4, 4), 100),
    (synth.Shape(1, 8, 2, 64, 1500, 2, 2), 128),
    (synth.Shape(1, 3, 3, 128, 1000, 2, 2), 20),
    (synth.Shape(1, 16, 2, 128, 777, 4, 4), 128),
    (synth.Shape(1, 7, 1, 128, 900, 4, 4), 64),
    (synth.Shape(1, 4, 1, 128, 1000, 4, 8), 128),
]


def _oracle_residual(x, seq_lens=None, res_lens=None):
    return oracle.decode_attention_residual(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"],
                                            x["k_res"], x["v_res"], seq_lens, res_lens)


@pytest.mark.parametrize("vname", list(VARIANTS))
@pytest.mark.parametrize("case", RESIDUAL, ids=lambda c: f"B{c[0].B}h{c[0].Hq}-{c[0].Hkv}D{c[0].D}N{c[0].N}R{c[1]}")
@pytest.mark.parametrize("splits", [1, 3])
def test_decode_residual_window(case, splits, vname):
    shape, R = case
    variant = VARIANTS[vname]
    if not _supported(shape, variant):
        pytest.skip("variant does not cover this configuration")
    x = synth.decode_inputs(shape, seed=shape.N + R)
    x.update(synth.residual_window(shape, seed=R, r_cap=R))
    ref = _oracle_residual(x)
    base = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    # the window must matter in this input: it holds a visible share of the softmax mass somewhere
    share = 1.0 - np.exp(base[1] - ref[1])
    assert share.max() > 1e-3
    got = gpu_decode_residual(shape, x, num_splits=splits, variant=variant)
    assert_decode_close(*got, *ref, what=f"{vname} R={R} splits={splits}")


def test_decode_residual_ragged_empty_parts_and_capacity():
    """Ragged code-cache and window lengths: a sequence with only a window, one with only codes,
    one with neither (o = 0, L = -inf); R below the window capacity."""
    shape = synth.Shape(4, 8, 2, 128, 640, 4, 4)
    x = synth.decode_inputs(shape, seed=21, n_cap=700)
    x.update(synth.residual_window(shape, seed=22, r_cap=128))
    seq = np.array([640, 0, 0, 333])
    res = np.array([100, 17, 0, 0])
    got_o, got_l = gpu_decode_residual(shape, x, seq_lens=seq, res_lens=res, N=640, R=100, num_splits=4)
    keep = [0, 1, 3]
    sub = {k: (v[keep] if k in ("q", "k_idx", "v_idx", "k_res", "v_res") else v) for k, v in x.items()}
    ref_o, ref_l = _oracle_residual(sub, seq[keep], res[keep])
    assert_decode_close(got_o[keep], got_l[keep], ref_o, ref_l, what="ragged residual")
    assert (got_o[2] == 0).all() and np.isneginf(got_l[2]).all()
    # rows at or beyond R are not attended even if res_lens says more
    got2 = gpu_decode_residual(shape, x, seq_lens=seq, res_lens=np.array([128, 128, 0, 0]), N=640, R=17)
    ref2 = _oracle_residual(sub, seq[keep], np.array([17, 17, 0]))
    assert_decode_close(got2[0][keep], got2[1][keep], *ref2, what="R clamps res_lens")


def test_decode_residual_without_code_cache_and_empty_window():
    shape = synth.Shape(2, 8, 2, 128, 256, 4, 4)
    x = synth.decode_inputs(shape, seed=23)
    x.update(synth.residual_window(shape, seed=24, r_cap=64))
    # N = 0: plain attention over the window
    got = gpu_decode_residual(shape, x, N=0)
    ref = _oracle_residual(x, seq_lens=np.zeros(2, dtype=np.int64))
    assert_decode_close(*got, *ref, what="window only")
    # R = 0: the same numbers as the call without a window
    got0 = gpu_decode_residual(shape, x, R=0, num_splits=2)
    base = gpu_decode(shape, x, num_splits=2)
    np.testing.assert_array_equal(got0[0], base[0])
    np.testing.assert_array_equal(got0[1], base[1])


def test_decode_residual_flush_then_attend():
    """Life cycle of the window: attend with it, then quantize it into the code cache
    (encode with pos0 = N) and attend without: the codes written are the oracle's."""
    shape = synth.Shape(1, 8, 2, 128, 512, 4, 4)
    R = 128
    x = synth.decode_inputs(shape, seed=25, n_cap=shape.N + R)
    x.update(synth.residual_window(shape, seed=26, r_cap=R))
    cfg = cfg_of(shape)
    k_idx, v_idx = dev(x["k_idx"]), dev(x["v_idx"])
    vb.vecinfer_encode_keys(cfg, dev(x["k_res"]), dev(x["lam"]), dev(x["cb_k"]), k_idx, pos0=shape.N)
    vb.vecinfer_encode_values(cfg, dev(x["v_res"]), dev(x["cb_v"]), v_idx, pos0=shape.N)
    torch.cuda.synchronize()
    ref_k, gap_k = oracle.encode_keys(x["k_res"], x["lam"], x["cb_k"], want_gap=True)
    ref_v, gap_v = oracle.encode_values(x["v_res"], x["cb_v"], want_gap=True)
    assert_indices_match(k_idx.cpu().numpy()[:, :, shape.N:], ref_k, gap_k, "flushed keys")
    assert_indices_match(v_idx.cpu().numpy()[:, :, shape.N:], ref_v, gap_v, "flushed values")
    np.testing.assert_array_equal(k_idx.cpu().numpy()[:, :, :shape.N], x["k_idx"][:, :, :shape.N])
    y = dict(x, k_idx=k_idx.cpu().numpy(), v_idx=v_idx.cpu().numpy())
    got = gpu_decode(shape, y)
    ref = oracle.decode_attention(y["q"], y["lam"], y["cb_k"], y["cb_v"], y["k_idx"], y["v_idx"])
    assert_decode_close(*got, *ref, what="after flush")


def test_decode_residual_full_size_196k():
    """The benchmark's launch configuration plus a full 128-row window."""
    shape = synth.LLAMA8B_196K
    x = synth.decode_inputs(shape, seed=4)
    x.update(synth.residual_window(shape, seed=27, r_cap=128))
    ref = _oracle_residual(x)
    got = gpu_decode_residual(shape, x)
    assert_decode_close(*got, *ref, what="196k + window")


# ------------------------------------------------------------------ fused decode step (Eq. 9 + Eq. 10)

def _new_token(shape, seed):
    g = synth.rng(seed)
    k, _ = synth.keys_with_outlier_channels(g, shape.B, shape.Hkv, 1, shape.D, 3)
    return k, synth.values(g, shape.B, shape.Hkv, 1, shape.D)


def _gpu_step(shape, x, k_new, v_new, seq_lens=None, N=None, num_splits=0, variant=vb.VARIANT_AUTO):
    cfg = cfg_of(shape)
    t = {k: dev(v) for k, v in x.items() if k in ("q", "lam", "cb_k", "cb_v", "k_idx", "v_idx")}
    B, n_cap = shape.B, x["k_idx"].shape[2]
    N = n_cap if N is None else N
    ws = vb.new_workspace(cfg, B, N, num_splits)
    out = torch.full((B, shape.Hq, shape.D), float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full((B, shape.Hq), float("nan"), dtype=torch.float32, device="cuda")
    sl = None if seq_lens is None else torch.as_tensor(np.asarray(seq_lens), dtype=torch.int32).cuda()
    vb.vecinfer_decode_step(cfg, t["q"], dev(k_new), dev(v_new), t["lam"], t["cb_k"], t["cb_v"], t["k_idx"],
                            t["v_idx"], ws, out, lse=lse, seq_lens=sl, N=N, num_splits=num_splits, variant=variant)
    torch.cuda.synchronize()
    return (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64),
            t["k_idx"].cpu().numpy(), t["v_idx"].cpu().numpy())


def _check_step(shape, x, k_new, v_new, got, lens, what):
    """Codes of the new token against the oracle's encode (near-ties logged), every other row
    untouched, and the attention against the oracle on the cache the step left behind."""
    out, lse, k_idx, v_idx = got
    ref_k, gap_k = oracle.encode_keys(k_new, x["lam"], x["cb_k"], want_gap=True)
    ref_v, gap_v = oracle.encode_values(v_new, x["cb_v"], want_gap=True)
    exp_k, exp_v = x["k_idx"].copy(), x["v_idx"].copy()
    for b in range(shape.B):
        if lens[b] == 0:
            continue
        pos = lens[b] - 1
        assert_indices_match(k_idx[b, :, pos], ref_k[b, :, 0], gap_k[b, :, 0], f"{what}: key codes b={b}")
        assert_indices_match(v_idx[b, :, pos], ref_v[b, :, 0], gap_v[b, :, 0], f"{what}: value codes b={b}")
        exp_k[b, :, pos] = k_idx[b, :, pos]
        exp_v[b, :, pos] = v_idx[b, :, pos]
    np.testing.assert_array_equal(k_idx, exp_k)          # no other row was written
    np.testing.assert_array_equal(v_idx, exp_v)
    keep = [b for b in range(shape.B) if lens[b] > 0]
    ref = oracle.decode_attention(x["q"][keep], x["lam"], x["cb_k"], x["cb_v"], k_idx[keep], v_idx[keep],
                                  np.asarray(lens)[keep])
    assert_decode_close(out[keep], lse[keep], *ref, what=what)
    for b in range(shape.B):
        if lens[b] == 0:
            assert (out[b] == 0).all() and np.isneginf(lse[b]).all()


STEP_SHAPES = [
    synth.Shape(2, 8, 2, 128, 777, 4, 4),
    synth.Shape(1, 8, 2, 128, 1500, 2, 2),
    synth.Shape(1, 4, 1, 128, 4099, 4, 4),
    synth.Shape(1, 4, 2, 64, 513, 4, 2),
    synth.Shape(1, 8, 1, 64, 300, 8, 8),
    synth.Shape(2, 8, 2, 64, 777, 4, 4),
    synth.Shape(1, 8, 2, 64, 1500, 2, 2),
    synth.Shape(2, 4, 2, 128, 777, 4, 4),
    synth.Shape(2, 2, 2, 64, 900, 4, 4),
    synth.Shape(2, 8, 2, 128, 777, 2, 4),
    synth.Shape(1, 8, 2, 128, 900, 4, 2),
    synth.Shape(1, 16, 2, 128, 777, 4, 4),
    synth.Shape(1, 7, 1, 64, 900, 4, 4),
    synth.Shape(2, 8, 2, 128, 777, 8, 8),
    synth.Shape(1, 8, 2, 64, 900, 8, 4),
]


@pytest.mark.parametrize("vname", list(VARIANTS))
@pytest.mark.parametrize("shape", STEP_SHAPES, ids=lambda s: f"B{s.B}h{s.Hq}-{s.Hkv}D{s.D}N{s.N}k{s.d_k}v{s.d_v}")
@pytest.mark.parametrize("splits", [1, 5, 64, 0])
def test_decode_step(shape, splits, vname):
    variant = VARIANTS[vname]
    if not _supported(shape, variant):
        pytest.skip("variant does not cover this configuration")
    x = synth.decode_inputs(shape, seed=shape.N + 31)
    k_new, v_new = _new_token(shape, seed=shape.N + 32)
    got = _gpu_step(shape, x, k_new, v_new, num_splits=splits, variant=variant)
    _check_step(shape, x, k_new, v_new, got, [shape.N] * shape.B, f"step {vname} S={splits}")


@pytest.mark.parametrize("vname", list(VARIANTS))
def test_decode_step_ragged_and_degenerate(vname):
    """Per-sequence append positions; a sequence whose only token is the new one; an empty one."""
    shape = synth.Shape(4, 8, 2, 128, 900, 4, 4)
    x = synth.decode_inputs(shape, seed=41, n_cap=1000)
    k_new, v_new = _new_token(shape, seed=42)
    lens = [900, 1, 0, 334]
    got = _gpu_step(shape, x, k_new, v_new, seq_lens=lens, N=900, num_splits=4, variant=VARIANTS[vname])
    _check_step(shape, x, k_new, v_new, got, lens, f"ragged step {vname}")


def test_decode_step_equals_append_then_attend():
    """The fused step writes exactly the codes of vecinfer_append_kv and returns the numbers of
    vecinfer_decode_attention on the result, up to the rounding of one more merged partial."""
    shape = synth.Shape(2, 8, 2, 128, 2049, 4, 4)
    x = synth.decode_inputs(shape, seed=43)
    k_new, v_new = _new_token(shape, seed=44)
    out, lse, k_idx, v_idx = _gpu_step(shape, x, k_new, v_new)
    cfg = cfg_of(shape)
    k2, v2 = dev(x["k_idx"]), dev(x["v_idx"])
    vb.vecinfer_append_kv(cfg, dev(k_new), dev(v_new), dev(x["lam"]), dev(x["cb_k"]), dev(x["cb_v"]), k2, v2,
                          pos0=shape.N - 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(k_idx, k2.cpu().numpy())
    np.testing.assert_array_equal(v_idx, v2.cpu().numpy())
    ref = gpu_decode(shape, dict(x, k_idx=k2, v_idx=v2))
    assert_decode_close(out, lse, *ref, what="fused vs separate")


def test_decode_step_full_size_196k():
    shape = synth.LLAMA8B_196K
    x = synth.decode_inputs(shape, seed=4)
    k_new, v_new = _new_token(shape, seed=45)
    got = _gpu_step(shape, x, k_new, v_new)
    _check_step(shape, x, k_new, v_new, got, [shape.N], "step 196k")


def test_decode_head_dim_64_long():
    """Head dim 64 (the paper's second kernel-sweep shape) at a length that gives every
    wavefront several tiles and uses the uneven tile deal: 32 / 8 heads, 65536 tokens."""
    shape = synth.Shape(1, 32, 8, 64, 65536, 4, 4)
    x = synth.decode_inputs(shape, seed=64)
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    got = gpu_decode(shape, x, variant=vb.VARIANT_MFMA)
    assert_decode_close(*got, *ref, what="D=64, 64k tokens")
    k_new, v_new = _new_token(shape, seed=65)
    step = _gpu_step(shape, x, k_new, v_new, variant=vb.VARIANT_MFMA)
    _check_step(shape, x, k_new, v_new, step, [shape.N], "step D=64, 64k tokens")


D64_DV8 = [synth.Shape(2, 8, 2, 64, 5000, 8, 8), synth.Shape(1, 6, 2, 64, 3333, 4, 8), synth.Shape(1, 16, 2, 64, 1111, 2, 8),
           synth.Shape(3, 2, 2, 64, 70, 8, 8)]


@pytest.mark.parametrize("shape", D64_DV8, ids=lambda s: f"B{s.B}h{s.Hq}-{s.Hkv}N{s.N}k{s.d_k}")
@pytest.mark.parametrize("splits", [1, 7, 0])
def test_decode_head_dim_64_value_sub_vectors_of_8(shape, splits):
    """D = 64 with d_v = 8 has 8 value sub-spaces for 16 matrix-core columns: the kernel handles each
    as two halves of 4 channels that share the code byte.  Attention, ragged lengths and the fused
    step against the oracle (Eq. 10, Eq. 9)."""
    x = synth.decode_inputs(shape, seed=shape.N + shape.d_k)
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    got = gpu_decode(shape, x, num_splits=splits, variant=vb.VARIANT_MFMA)
    assert_decode_close(*got, *ref, what=f"D=64 d_v=8 S={splits}")
    k_new, v_new = _new_token(shape, seed=shape.N + 9)
    step = _gpu_step(shape, x, k_new, v_new, num_splits=splits, variant=vb.VARIANT_MFMA)
    _check_step(shape, x, k_new, v_new, step, [shape.N] * shape.B, f"step D=64 d_v=8 S={splits}")
    if shape.B > 1:
        lens = [shape.N // 3, 0, 1][:shape.B]
        k_new, v_new = _new_token(shape, seed=shape.N + 10)
        step = _gpu_step(shape, x, k_new, v_new, seq_lens=lens, N=shape.N, num_splits=splits, variant=vb.VARIANT_MFMA)
        _check_step(shape, x, k_new, v_new, step, lens, f"ragged step D=64 d_v=8 S={splits}")


# ------------------------------------------------------------------ K-Means codebook training step

def _gpu_kmeans(shape, x, lam, cb):
    cfg = cfg_of(shape)
    keys = lam is not None
    d = shape.d_k if keys else shape.d_v
    M = shape.D // d
    B, Hkv, T, _ = x.shape
    cb_out = torch.full((Hkv, M, 256, d), float("nan"), dtype=torch.float16, device="cuda")
    codes = torch.full((B, Hkv, T, M), 0xEE, dtype=torch.uint8, device="cuda")
    counts = torch.full((Hkv, M, 256), -1, dtype=torch.int32, device="cuda")
    ws = vb.new_kmeans_workspace(cfg, keys)
    vb.vecinfer_kmeans_step(cfg, dev(x), None if lam is None else dev(lam), dev(cb), cb_out, codes, ws, counts=counts)
    torch.cuda.synchronize()
    return cb_out.cpu().numpy(), codes.cpu().numpy(), counts.cpu().numpy()


def _check_kmeans(shape, x, lam, cb, got, what):
    """Assignment against the oracle's Eq. 2 (near-ties logged); update against the oracle's means
    for the assignment the GPU made (fp32 sums, fp16 result: one fp16 ulp)."""
    cb_out, codes, counts = got
    B, Hkv, T, D = x.shape
    if lam is not None:
        ref_idx, gap = oracle.encode_keys(x, lam, cb, want_gap=True)
    else:
        ref_idx, gap = oracle.encode_values(x, cb, want_gap=True)
    assert_indices_match(codes, ref_idx, gap, f"{what}: assignment")
    for g in range(Hkv):
        rows = x[:, g].reshape(B * T, D).astype(np.float64)
        if lam is not None:
            rows = oracle.transform_keys(rows, lam[g])
        ref_cb, ref_counts = oracle.kmeans_update(rows, codes[:, g].reshape(B * T, -1), cb[g])
        np.testing.assert_array_equal(counts[g], ref_counts)
        np.testing.assert_allclose(cb_out[g].astype(np.float64), ref_cb, rtol=1.5e-3, atol=1e-6,
                                   err_msg=f"{what}: centroids of head {g}")
        empty = ref_counts == 0
        np.testing.assert_array_equal(cb_out[g][empty], cb[g][empty])     # untouched, bit for bit


@pytest.mark.parametrize("kind", ["keys", "values"])
@pytest.mark.parametrize("shape", [synth.Shape(2, 4, 2, 128, 1000, 4, 4), synth.Shape(1, 2, 2, 64, 777, 2, 8),
                                   synth.Shape(3, 1, 1, 128, 70, 8, 2)],
                         ids=lambda s: f"B{s.B}g{s.Hkv}D{s.D}T{s.N}k{s.d_k}v{s.d_v}")
def test_kmeans_step(shape, kind):
    e = synth.encode_inputs(shape, seed=shape.N + 7, n_outlier=3)
    if kind == "keys":
        lam = np.stack([oracle.smoothing_factors(e["k"][:, h]) for h in range(shape.Hkv)]).astype(np.float32)
        x, cb = e["k"], e["cb_k"]
    else:
        lam, x, cb = None, e["v"], e["cb_v"]
    cb = cb.copy()
    cb[:, :, 9] = 300.0                                   # a centroid nobody is assigned to
    got = _gpu_kmeans(shape, x, lam, cb)
    _check_kmeans(shape, x, lam, cb, got, f"kmeans {kind}")


def test_kmeans_iterations_reduce_the_quantization_error():
    """A few Lloyd iterations on the GPU: the error of the codebook (measured by the oracle) goes
    down monotonically (up to the fp16 rounding of the centroids)."""
    shape = synth.Shape(2, 2, 2, 128, 2048, 4, 4)
    e = synth.encode_inputs(shape, seed=71, n_outlier=3)
    x = e["v"]
    cb = e["cb_v"]

    def error(cbx):
        idx = oracle.encode_values(x, cbx)
        tot = 0.0
        for g in range(shape.Hkv):
            rows = x[:, g].reshape(-1, shape.D).astype(np.float64)
            tot += ((rows - oracle.vq_dequantize(idx[:, g].reshape(rows.shape[0], -1), cbx[g])) ** 2).sum()
        return tot

    errs = [error(cb)]
    for _ in range(4):
        cb, _, counts = _gpu_kmeans(shape, x, None, cb)
        assert counts.sum() == shape.Hkv * shape.Mv * shape.B * shape.N
        errs.append(error(cb))
    assert all(b <= a * (1 + 1e-3) for a, b in zip(errs, errs[1:])), errs
    assert errs[-1] < 0.8 * errs[0]


# ------------------------------------------------------------------ smoothing-factor calibration (Eq. 4)

@pytest.mark.parametrize("shape", [synth.Shape(3, 4, 2, 128, 700, 4, 4), synth.Shape(1, 8, 8, 64, 1, 4, 4),
                                   synth.Shape(2, 2, 1, 128, 513, 8, 8, 12, 12)],
                         ids=lambda s: f"B{s.B}g{s.Hkv}D{s.D}T{s.N}")
def test_calibrate_lambda(shape):
    """lambda = sqrt(max |K|) per (KV head, channel) over every token of every sequence; the maximum
    is exact, the square root is one fp32 rounding; an all-zero channel gets the floor."""
    k, _ = synth.keys_with_outlier_channels(synth.rng(shape.N + 3), shape.B, shape.Hkv, shape.N, shape.D, 3)
    k[:, 0, :, 5] = 0                                         # a channel with no signal at all
    lam = torch.full((shape.Hkv, shape.D), float("nan"), dtype=torch.float32, device="cuda")
    vb.vecinfer_calibrate_lambda(cfg_of(shape), dev(k), lam)
    torch.cuda.synchronize()
    got = lam.cpu().numpy()
    ref = np.stack([oracle.smoothing_factors(k[:, h]) for h in range(shape.Hkv)])
    assert ref[0, 5] == 0 and got[0, 5] == np.float32(vb.LAMBDA_FLOOR)
    ref[0, 5] = vb.LAMBDA_FLOOR
    np.testing.assert_allclose(got, ref, rtol=1.2e-7, atol=0)
    # the calibrated factors are usable as they are: encode with them and compare with the oracle
    if shape.b_k == 8 and shape.N > 1:
        cb = synth.codebooks(synth.rng(1), shape.Hkv, shape.Mk, shape.d_k)
        (got_k,) = gpu_encode(shape, k=k, lam=got, cb_k=cb)
        ref_k, gap = oracle.encode_keys(k, got, cb, want_gap=True)
        assert_indices_match(got_k, ref_k, gap, "encode with calibrated lambda")


# ------------------------------------------------------------------ the longest cache the matrix-core path takes

def test_decode_at_the_maximum_length():
    """N just under the 32-bit row-offset limit (N * D / 2 < 2^31: 33.5 M tokens at D = 128, 1 GiB of
    codes per side).  The bulk of the cache is one repeated token (every code 7), the last 3000
    tokens are random: the oracle attends to the tail, the bulk has the closed form
    L = s_0 + ln N_0, o = its one value row, and the two are joined by the log-sum-exp merge.
    The query is scaled so that bulk and tail weigh about the same: a wrong offset anywhere near
    the end of the buffers, or a lost stretch of the bulk, changes the result."""
    shape = synth.Shape(1, 1, 1, 128, (1 << 25) - 5, 4, 4)
    tail = 3000
    x = synth.decode_inputs(synth.Shape(1, 1, 1, 128, tail, 4, 4), seed=99)
    N0 = shape.N - tail
    one = np.full((1, 1, 1, 32), 7, dtype=np.uint8)

    def parts(scale):
        q = (x["q"].astype(np.float32) * scale).astype(np.float16)
        t_o, t_l = oracle.decode_attention(q, x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
        b_o, b_l = oracle.decode_attention(q, x["lam"], x["cb_k"], x["cb_v"], one, one)       # a single token
        return q, t_o, t_l, b_o, b_l + np.log(N0)

    lo, hi = 0.0, 16.0                         # tail log-weight minus bulk log-weight grows with the scale
    for _ in range(30):
        mid = 0.5 * (lo + hi)
        _, _, t_l, _, b_l = parts(mid)
        lo, hi = (mid, hi) if t_l[0, 0] < b_l[0, 0] else (lo, mid)
    q, t_o, t_l, b_o, b_l = parts(hi)
    ref_o, ref_l = oracle.merge_splits(np.stack([b_o[0, 0], t_o[0, 0]]), np.array([b_l[0, 0], t_l[0, 0]]))
    share = np.exp(t_l[0, 0] - ref_l)          # weight of the tail in the softmax
    assert 0.2 < share < 0.8, share

    k_idx = torch.full((1, 1, shape.N, 32), 7, dtype=torch.uint8, device="cuda")
    v_idx = torch.full((1, 1, shape.N, 32), 7, dtype=torch.uint8, device="cuda")
    k_idx[:, :, N0:] = dev(x["k_idx"])
    v_idx[:, :, N0:] = dev(x["v_idx"])
    got_o, got_l = gpu_decode(shape, dict(x, q=q, k_idx=k_idx, v_idx=v_idx), variant=vb.VARIANT_MFMA)
    assert_decode_close(got_o, got_l, ref_o[None, None], np.array([[ref_l]]), what="N = 2^25 - 5")
    del k_idx, v_idx
    # one token more than the limit is refused by this variant, not mis-addressed
    cfg = cfg_of(shape)
    n_big = 1 << 25
    ws = vb.new_workspace(cfg, 1, n_big)
    out = torch.empty((1, 1, 128), dtype=torch.float16, device="cuda")
    kb = torch.empty((1, 1, n_big, 32), dtype=torch.uint8, device="cuda")
    with pytest.raises(vb.VecInferError) as e:
        vb.vecinfer_decode_attention(cfg, dev(q), dev(x["lam"]), dev(x["cb_k"]), dev(x["cb_v"]), kb, kb, ws, out,
                                     variant=vb.VARIANT_MFMA)
    assert e.value.code == vb.EUNSUPPORTED
