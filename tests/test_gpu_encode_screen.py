"""The cache-fill search on inputs chosen against its matrix-core screen (Eq. 2: the code is the
nearest centroid by the fp32 direct distance, lowest index among equals; the screen may only
shortlist).  Planted exact ties, duplicated and one-ulp-apart centroids, tiny and huge scales,
values that overflow the screen's fp16 operands (plain-search fallback), all against the oracle's
argmin (bit-exact except logged near-ties) or against the tie rule itself where the arithmetic is
exact."""
import numpy as np
import pytest

import oracle
from paper_2510_06175_amd import synth

from helpers import assert_indices_match, gpu_encode

pytestmark = pytest.mark.gpu

T = 200          # > 64: the tiled kernel (the per-token kernel serves short inputs)


def _values_case(D, d, x, cb):
    """x [T, D] fp16, cb [M, 256, d] fp16 -> (GPU codes [T, M], oracle codes, oracle gap)."""
    shape = synth.Shape(1, 1, 1, D, x.shape[0], d, d)
    got, = gpu_encode(shape, v=x[None, None], cb_v=cb[None])
    ref, gap = oracle.encode_values(x[None, None], cb[None], want_gap=True)
    return got[0, 0], ref[0, 0], gap[0, 0]


@pytest.mark.parametrize("d", [2, 4, 8])
@pytest.mark.parametrize("D", [64, 128])
def test_exact_ties_go_to_the_lowest_index(D, d):
    """Centroids on a grid of small integers / 2 and tokens at centroids and at midpoints between two
    of them: every distance is exact in fp32, so ties are exact and the lower index must win."""
    g = synth.rng(D + d)
    M = D // d
    cb = (g.integers(-8, 9, size=(M, 256, d)) / 2).astype(np.float16)
    cb[:, 200] = cb[:, 13]                                   # duplicates: 13 must win over 200
    cb[:, 255] = cb[:, 0]
    a = g.integers(0, 256, size=(T, M))
    b = g.integers(0, 256, size=(T, M))
    pick = lambda idx: np.take_along_axis(cb[None].repeat(T, 0), idx[:, :, None, None].repeat(d, 3), 2)[:, :, 0]
    x = ((pick(a).astype(np.float32) + pick(b).astype(np.float32)) / 2).astype(np.float16)   # midpoints: exact in fp16
    x[::3] = pick(a)[::3]                                    # every third token sits on a centroid
    x = x.reshape(T, D)
    got, ref, gap = _values_case(D, d, x, cb)
    xs = x.reshape(T, M, 1, d).astype(np.float64)
    dist = ((xs - cb[None].astype(np.float64)) ** 2).sum(-1)              # exact (halves of small integers)
    want = dist.argmin(-1)                                                # numpy: first minimum = lowest index
    np.testing.assert_array_equal(got, want)
    assert ((dist == dist.min(-1, keepdims=True)).sum(-1) > 1).mean() > 0.005   # the case does hold ties


@pytest.mark.parametrize("scale_x,scale_c", [(1e-3, 1e-3), (1.0, 1e-3), (1e-3, 1.0), (30.0, 30.0), (200.0, 1.0),
                                             (1.0, 150.0)])
@pytest.mark.parametrize("d", [2, 4, 8])
def test_scales(d, scale_x, scale_c):
    """Tokens and centroids from 1e-3 to 200 in size, together and against each other (the screen
    scales its operands per sub-space; what it cannot represent falls back to the plain search)."""
    D = 128
    g = synth.rng(int(scale_x * 1000) + int(scale_c * 1000) + d)
    M = D // d
    cb = (g.standard_normal((M, 256, d)) * scale_c).astype(np.float16)
    x = (g.standard_normal((T, D)) * scale_x).astype(np.float16)
    got, ref, gap = _values_case(D, d, x, cb)
    assert_indices_match(got, ref, gap, f"scales d={d} x{scale_x} c{scale_c}")


@pytest.mark.parametrize("d", [2, 4, 8])
def test_one_ulp_neighbours_and_fp16_extremes(d):
    """Pairs of centroids one fp16 ulp apart with tokens next to them; tokens at the largest fp16
    values (the screen's scaled operands overflow: plain search); an all-zero codebook sub-space."""
    D = 128
    g = synth.rng(77 + d)
    M = D // d
    cb = g.standard_normal((M, 256, d)).astype(np.float16)
    nxt = np.nextafter(cb[:, :128].astype(np.float16), np.float16(np.inf)).astype(np.float16)
    cb[:, 128:] = nxt                                        # centroid 128 + i = centroid i, one ulp up
    cb[3] = 0                                                # a sub-space whose centroids are all zero
    a = g.integers(0, 256, size=(T, M))
    x = np.take_along_axis(cb[None].repeat(T, 0), a[:, :, None, None].repeat(d, 3), 2)[:, :, 0].astype(np.float32)
    x += g.standard_normal(x.shape).astype(np.float32) * 1e-3
    x = x.astype(np.float16).reshape(T, D)
    x[5] = 65504.0
    x[6] = -65504.0
    x[7, ::2] = 60000.0
    got, ref, gap = _values_case(D, d, x, cb)
    assert (got[:, 3] == 0).all()                            # all centroids equal: index 0
    keep = np.ones(T, bool)
    keep[[5, 6, 7]] = False                                  # (their fp64 distances tie far below fp32 resolution)
    assert_indices_match(got[keep], ref[keep], gap[keep], f"ulp neighbours d={d}")
    # the extreme rows against the rule in fp32 itself
    cb32 = cb.astype(np.float32)
    for t in (5, 6, 7):
        xs = x[t].astype(np.float32).reshape(M, 1, d)
        dist = np.zeros((M, 256), np.float32)
        for j in range(d):
            diff = xs[:, :, j] - cb32[:, :, j]
            dist = (diff * diff + dist).astype(np.float32) if j else (diff * diff).astype(np.float32)
        # fp32 fused multiply-add differs from multiply-then-add in the last bit: accept any centroid
        # whose distance is within 2 ulp of the minimum, and require the exact one where it is alone
        best = dist.min(-1, keepdims=True)
        ok = dist <= best * (1 + 3e-7)
        assert ok[np.arange(M), got[t]].all()


def test_keys_with_outliers_full_tile_mix():
    """The key path (smoothing + Hadamard in front of the search) at a length with a ragged tail,
    several sequences and KV heads, outlier channels x20."""
    shape = synth.Shape(2, 4, 2, 128, 333, 4, 4)
    e = synth.encode_inputs(shape, seed=9, n_outlier=4)
    lam = np.stack([oracle.smoothing_factors(e["k"][:, h]) for h in range(shape.Hkv)]).astype(np.float32)
    got, = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"])
    ref, gap = oracle.encode_keys(e["k"], lam, e["cb_k"], want_gap=True)
    assert_indices_match(got, ref, gap, "keys with outliers")


# ------------------------------------------------------------------ shared codebooks (10- / 12-bit codes)

def _wide_values_case(D, d, bits, x, cb):
    """x [T, D] fp16, cb [2^bits, d] fp16 -> (GPU codes [T, M], oracle codes, oracle gap)."""
    shape = synth.Shape(1, 1, 1, D, x.shape[0], d, d, bits, bits)
    got, = gpu_encode(shape, v=x[None, None], cb_v=cb[None])
    ref, gap = oracle.encode_values(x[None, None], cb[None, None], want_gap=True)
    return oracle.unpack_codes(got, bits, D // d)[0, 0], ref[0, 0], gap[0, 0]


@pytest.mark.parametrize("D,d,bits", [(128, 8, 12), (128, 4, 12), (128, 4, 10), (64, 8, 12), (64, 4, 10)])
def test_shared_codebook_exact_ties_across_chunks(D, d, bits):
    """A table of 2^b centroids that holds only 40 different vectors on a grid of halves: every
    token's nearest centroid occurs about 2^b / 40 times, spread over all 256-centroid chunks of the
    search, all at exactly the same distance.  More than two chunks tie, so the screen gives up and
    the plain search must return the lowest index."""
    g = synth.rng(D + d + bits)
    C = 1 << bits
    M = D // d
    base = (g.integers(-6, 7, size=(40, d)) / 2).astype(np.float16)
    cb = base[g.integers(0, 40, size=C)]
    x = (base[g.integers(0, 40, size=(T, M))].astype(np.float32)
         + g.integers(-1, 2, size=(T, M, d)).astype(np.float32) / 4).astype(np.float16).reshape(T, D)
    got, ref, gap = _wide_values_case(D, d, bits, x, cb)
    dist = ((x.reshape(T, M, 1, d).astype(np.float64) - cb[None, None].astype(np.float64)) ** 2).sum(-1)   # exact
    np.testing.assert_array_equal(got, dist.argmin(-1))
    assert ((dist == dist.min(-1, keepdims=True)).sum(-1) > 2).mean() > 0.9


@pytest.mark.parametrize("scale", [1e-3, 1.0, 100.0])
@pytest.mark.parametrize("D,d,bits", [(128, 8, 12), (128, 4, 10), (64, 4, 12)])
def test_shared_codebook_scales_and_near_ties(D, d, bits, scale):
    """Random shared tables at three scales with a block of centroids one fp16 ulp above others (in
    other chunks), tokens near centroids, and tokens at the largest fp16 values."""
    g = synth.rng(int(scale * 1000) + D + d + bits)
    C = 1 << bits
    M = D // d
    cb = (g.standard_normal((C, d)) * scale).astype(np.float16)
    cb[C // 2:C // 2 + 300] = np.nextafter(cb[:300], np.float16(np.inf)).astype(np.float16)
    a = g.integers(0, C, size=(T, M))
    x = cb[a].astype(np.float32) * (1 + g.standard_normal((T, M, d)).astype(np.float32) * 1e-3)
    x = x.astype(np.float16).reshape(T, D)
    x[11] = 65504.0
    x[12, ::3] = -60000.0
    got, ref, gap = _wide_values_case(D, d, bits, x, cb)
    keep = np.ones(T, bool)
    keep[[11, 12]] = False                                  # (fp64 gaps far below fp32 resolution there)
    assert_indices_match(got[keep], ref[keep], gap[keep], f"shared table d{d}b{bits} x{scale}")
    cb32 = cb.astype(np.float32)
    for t in (11, 12):
        xs = x[t].astype(np.float32).reshape(M, 1, d)
        dist = ((xs - cb32[None]) ** 2).sum(-1, dtype=np.float32)
        best = dist.min(-1, keepdims=True)
        assert (dist[np.arange(M), got[t]] <= best[:, 0] * (1 + 1e-6)).all()
