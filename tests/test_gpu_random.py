"""GPU parity on seeded random configurations: every supported head dim, GQA group, sub-vector
dim and code width (8-bit per-sub-space tables, 10- / 12-bit shared tables), ragged batches, split
counts, cache-fill lengths and offsets.  Through the C ABI, against the float64 oracle."""
import numpy as np
import pytest

import oracle
from paper_2510_06175_amd import synth

from helpers import (assert_decode_close, assert_indices_match, gpu_decode, gpu_encode, oracle_view,
                     tile_value_codes)

pytestmark = pytest.mark.gpu


def _id(s):
    return f"B{s.B}h{s.Hq}-{s.Hkv}N{s.N}k{s.d_k}b{s.b_k}v{s.d_v}b{s.b_v}"


def _oracle_decode(shape, x, seq_lens=None):
    y = oracle_view(shape, x)
    return oracle.decode_attention(y["q"], y["lam"], y["cb_k"], y["cb_v"], y["k_idx"], y["v_idx"], seq_lens)


# ------------------------------------------------------------------ seeded random sweep over the whole configuration space

def _random_cases(n, seed):
    """Seeded random configurations: head dim, GQA group, sub-vector dims, code widths, batch,
    lengths (ragged, with tails that are not a multiple of any tile), split counts."""
    g = synth.rng(seed)
    sides = [(2, 8), (4, 8), (8, 8), (4, 10), (4, 12), (8, 10), (8, 12)]
    cases = []
    while len(cases) < n:
        D = int(g.choice([64, 128]))
        (dk, bk), (dv, bv) = sides[int(g.integers(len(sides)))], sides[int(g.integers(len(sides)))]
        wide = bk != 8 or bv != 8
        if wide and (dk < 4 or dv < 4):
            continue
        if D == 64 and ((dk, bk) == (8, 10) or (dv, bv) == (8, 10)):      # 10-byte rows: not supported
            continue
        G = int(g.choice([1, 2, 3, 4, 5, 8]))
        Hkv = int(g.choice([1, 2, 3]))
        B = int(g.choice([1, 2, 3]))
        N = int(g.integers(1, 2500))
        S = int(g.choice([0, 1, 2, 3, 7, 32]))
        lens = [int(g.integers(0, N + 1)) for _ in range(B)] if g.random() < 0.5 else None
        cases.append((synth.Shape(B, G * Hkv, Hkv, D, N, dk, dv, bk, bv), S, lens, int(g.integers(1 << 30))))
    return cases


@pytest.mark.parametrize("case", _random_cases(48, seed=2024),
                         ids=lambda c: f"{_id(c[0])}D{c[0].D}S{c[1]}{'r' if c[2] else ''}")
def test_decode_random_configurations(case):
    shape, S, lens, seed = case
    x = synth.decode_inputs(shape, seed=seed)
    got_o, got_l = gpu_decode(shape, x, seq_lens=lens, num_splits=S)
    lens_a = np.full(shape.B, shape.N) if lens is None else np.asarray(lens)
    keep = [b for b in range(shape.B) if lens_a[b] > 0]
    for b in range(shape.B):
        if lens_a[b] == 0:
            assert (got_o[b] == 0).all() and np.isneginf(got_l[b]).all()
    if keep:
        sub = {k: (v[keep] if k in ("q", "k_idx", "v_idx") else v) for k, v in x.items()}
        ref_o, ref_l = _oracle_decode(shape, sub, lens_a[keep])
        assert_decode_close(got_o[keep], got_l[keep], ref_o, ref_l, what=f"random {_id(shape)} S={S}")
    if shape.b_k == 8 and shape.b_v == 8 and shape.Mv >= 16:
        # the tiled layout of the value codes feeds the same arithmetic: same bits out
        cap = (shape.N + 63) // 64 * 64
        x2 = synth.decode_inputs(shape, seed=seed + 1, n_cap=cap)
        rows = gpu_decode(shape, x2, seq_lens=lens, N=shape.N, num_splits=S)
        tiled = gpu_decode(shape, dict(x2, v_idx=tile_value_codes(x2["v_idx"])), seq_lens=lens, N=shape.N,
                           num_splits=S, v_tiled=1)
        np.testing.assert_array_equal(tiled[0], rows[0])
        np.testing.assert_array_equal(tiled[1], rows[1])


def _random_encode_cases(n, seed):
    g = synth.rng(seed)
    sides = [(2, 8), (4, 8), (8, 8), (4, 10), (4, 12), (8, 10), (8, 12)]
    cases = []
    while len(cases) < n:
        D = int(g.choice([64, 128]))
        (dk, bk), (dv, bv) = sides[int(g.integers(len(sides)))], sides[int(g.integers(len(sides)))]
        if (bk != 8 or bv != 8) and (dk < 4 or dv < 4):
            continue
        if D == 64 and ((dk, bk) == (8, 10) or (dv, bv) == (8, 10)):      # 10-byte rows: not supported
            continue
        T = int(g.choice([1, 2, 15, 16, 17, 63, 64, 65, 200, 333]))
        cases.append((synth.Shape(int(g.choice([1, 2])), 2, int(g.choice([1, 2])), D, T, dk, dv, bk, bv),
                      int(g.integers(0, 40)), int(g.integers(1 << 30))))
    return cases


@pytest.mark.parametrize("case", _random_encode_cases(24, seed=77),
                         ids=lambda c: f"{_id(c[0])}D{c[0].D}T{c[0].N}p{c[1]}")
def test_encode_random_configurations(case):
    """Cache fill at random shapes, lengths around the kernels' switch-over points (16 / 17 tokens,
    64-token tiles) and offsets: codes against the oracle, untouched rows stay untouched."""
    shape, pos0, seed = case
    shape = synth.Shape(shape.B, 2 * shape.Hkv, shape.Hkv, shape.D, shape.N, shape.d_k, shape.d_v, shape.b_k, shape.b_v)
    e = synth.encode_inputs(shape, seed=seed, n_outlier=3)
    lam = synth.lognormal_lambda(synth.rng(seed + 1), shape.Hkv, shape.D)
    cap = pos0 + shape.N + 5
    got_k, got_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"], pos0=pos0, n_cap=cap)
    y = oracle_view(shape, {"cb_k": e["cb_k"], "cb_v": e["cb_v"]})
    ref_k, gap_k = oracle.encode_keys(e["k"], lam, y["cb_k"], want_gap=True)
    ref_v, gap_v = oracle.encode_values(e["v"], y["cb_v"], want_gap=True)
    rows = slice(pos0, pos0 + shape.N)
    assert_indices_match(oracle.unpack_codes(got_k[:, :, rows], shape.b_k, shape.Mk), ref_k, gap_k, "random keys")
    assert_indices_match(oracle.unpack_codes(got_v[:, :, rows], shape.b_v, shape.Mv), ref_v, gap_v, "random values")
    for got in (got_k, got_v):
        assert (got[:, :, :pos0] == 0xEE).all() and (got[:, :, pos0 + shape.N:] == 0xEE).all()


# ------------------------------------------------------------------ every instantiation of the attention kernel

def _all_side_combinations():
    """Every (head dim, key side, value side) the matrix-core kernel is built for, each with one
    head group (G = 4) and with two (G = 8): 2 x the 8-bit mixes + the 10- / 12-bit ones."""
    sides = [(2, 8), (4, 8), (8, 8), (4, 10), (4, 12), (8, 10), (8, 12)]
    cases = []
    for D in (64, 128):
        for dk, bk in sides:
            for dv, bv in sides:
                wide = bk != 8 or bv != 8
                if wide and (dk < 4 or dv < 4):
                    continue
                if D == 64 and ((dk, bk) == (8, 10) or (dv, bv) == (8, 10)):      # 10-byte rows: not supported
                    continue
                for G in (4, 8):
                    cases.append(synth.Shape(1, G, 1, D, 200, dk, dv, bk, bv))
    return cases


@pytest.mark.parametrize("shape", _all_side_combinations(), ids=lambda s: f"D{s.D}G{s.Hq}k{s.d_k}b{s.b_k}v{s.d_v}b{s.b_v}")
def test_every_side_combination(shape):
    """One small decode (200 tokens: three tiles and a tail, two splits) per instantiation of the
    attention kernel with value codes in rows, against the oracle."""
    seed = 31 * shape.D + 7 * shape.d_k + 5 * shape.d_v + shape.b_k + 3 * shape.b_v + shape.Hq
    x = synth.decode_inputs(shape, seed=seed)
    got_o, got_l = gpu_decode(shape, x, num_splits=2)
    ref_o, ref_l = _oracle_decode(shape, x)
    assert_decode_close(got_o, got_l, ref_o, ref_l, what=f"every combination {_id(shape)} D{shape.D}")


@pytest.mark.parametrize("shape", _all_side_combinations(), ids=lambda s: f"D{s.D}G{s.Hq}k{s.d_k}b{s.b_k}v{s.d_v}b{s.b_v}")
def test_every_side_combination_fused_step(shape):
    """The whole step (Eq. 9 + Eq. 10 in one call) per instantiation: the new token's codes must be
    what vecinfer_append_kv writes, bit for bit, and the output the oracle's on the cache with them."""
    import torch
    from paper_2510_06175_amd import binding as vb
    from helpers import cfg_of, dev
    seed = 17 * shape.D + 3 * shape.d_k + 11 * shape.d_v + shape.b_k + 5 * shape.b_v + shape.Hq
    N = shape.N
    x = synth.decode_inputs(shape, seed=seed, n_cap=N + 4)
    g = synth.rng(seed + 1)
    k_new, _ = synth.keys_with_outlier_channels(g, shape.B, shape.Hkv, 1, shape.D, 3)
    v_new = synth.values(g, shape.B, shape.Hkv, 1, shape.D)
    cfg = cfg_of(shape)
    t = {k: dev(v) for k, v in x.items()}
    ws = vb.new_workspace(cfg, shape.B, N, 3)
    out = torch.full((shape.B, shape.Hq, shape.D), float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full((shape.B, shape.Hq), float("nan"), dtype=torch.float32, device="cuda")
    vb.vecinfer_decode_step(cfg, t["q"], dev(k_new), dev(v_new), t["lam"], t["cb_k"], t["cb_v"], t["k_idx"],
                            t["v_idx"], ws, out, lse=lse, N=N, num_splits=3)
    torch.cuda.synchronize()
    k2, v2 = dev(x["k_idx"]), dev(x["v_idx"])
    vb.vecinfer_append_kv(cfg, dev(k_new), dev(v_new), t["lam"], t["cb_k"], t["cb_v"], k2, v2, pos0=N - 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t["k_idx"].cpu().numpy(), k2.cpu().numpy())
    np.testing.assert_array_equal(t["v_idx"].cpu().numpy(), v2.cpu().numpy())
    got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
    ref = _oracle_decode(shape, dict(x, k_idx=k2.cpu().numpy()[:, :, :N], v_idx=v2.cpu().numpy()[:, :, :N]))
    assert_decode_close(*got, *ref, what=f"fused step, every combination {_id(shape)} D{shape.D}")


def _all_tiled_combinations():
    return [synth.Shape(1, G, 1, D, 200, dk, dv) for D in (64, 128) for dk in (2, 4, 8) for dv in (2, 4, 8)
            if D // dv >= 16 for G in (4, 8)]


@pytest.mark.parametrize("shape", _all_tiled_combinations(), ids=lambda s: f"D{s.D}G{s.Hq}k{s.d_k}v{s.d_v}")
def test_every_tiled_instantiation(shape):
    """Every instantiation of the attention kernel for tiled value codes: the same bits out as with
    the codes in rows (which test_every_side_combination holds against the oracle)."""
    seed = 13 * shape.D + 3 * shape.d_k + 7 * shape.d_v + shape.Hq
    x = synth.decode_inputs(shape, seed=seed, n_cap=256)
    rows = gpu_decode(shape, x, N=shape.N, num_splits=2)
    tiled = gpu_decode(shape, dict(x, v_idx=tile_value_codes(x["v_idx"])), N=shape.N, num_splits=2, v_tiled=1)
    np.testing.assert_array_equal(tiled[0], rows[0])
    np.testing.assert_array_equal(tiled[1], rows[1])
    ref_o, ref_l = _oracle_decode(shape, dict(x, k_idx=x["k_idx"][:, :, :shape.N], v_idx=x["v_idx"][:, :, :shape.N]))
    assert_decode_close(*rows, ref_o, ref_l, what=f"tiled instantiation {_id(shape)} D{shape.D}")


def _all_encode_combinations():
    sides = [(2, 8), (4, 8), (8, 8), (4, 10), (4, 12), (8, 10), (8, 12)]
    return [(synth.Shape(1, 2, 1, D, T, d, d, b, b), 3, 1000 * D + 100 * d + b + T)
            for D in (64, 128) for d, b in sides if not (D == 64 and (d, b) == (8, 10)) for T in (5, 200)]


@pytest.mark.parametrize("case", _all_encode_combinations(),
                         ids=lambda c: f"D{c[0].D}d{c[0].d_k}b{c[0].b_k}T{c[0].N}")
def test_every_cache_fill_instantiation(case):
    """Every (head dim, sub-vector dim, code width) of the cache fill, keys and values, by the
    per-token kernel (5 tokens) and the tile kernel (200 tokens), against the oracle."""
    test_encode_random_configurations(case)
