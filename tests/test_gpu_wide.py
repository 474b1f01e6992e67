"""GPU parity for codes wider than 8 bits (d8b12, d4b12, d4b10, d8b10 and their mixes with 8-bit
sides; Sec. 4.1): one codebook of 2^b centroids per KV head shared by its sub-spaces (Sec. 2.2,
Alg. 1), token rows packed b bits per code.  Through the C ABI, against the float64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_06175_amd import binding as vb
from paper_2510_06175_amd import synth

from helpers import (assert_decode_close, assert_indices_match, cfg_of, dev, gpu_decode, gpu_decode_residual,
                     gpu_encode, oracle_view)

pytestmark = pytest.mark.gpu


def _id(s):
    return f"B{s.B}h{s.Hq}-{s.Hkv}N{s.N}k{s.d_k}b{s.b_k}v{s.d_v}b{s.b_v}"


def _oracle_decode(shape, x, seq_lens=None):
    y = oracle_view(shape, x)
    return oracle.decode_attention(y["q"], y["lam"], y["cb_k"], y["cb_v"], y["k_idx"], y["v_idx"], seq_lens)


# ------------------------------------------------------------------ decode

WIDE = [
    # B, Hq, Hkv, D, N, d_k, d_v, b_k, b_v  (several tiles and a ragged tail; G = 4, 1, 8, 3)
    synth.Shape(2, 8, 2, 128, 777, 8, 8, 12, 12),         # d8b12 (1.5 bits per element)
    synth.Shape(1, 4, 1, 128, 4099, 8, 8, 12, 12),
    synth.Shape(1, 16, 2, 128, 600, 8, 8, 12, 12),        # G = 8
    synth.Shape(2, 8, 2, 128, 900, 4, 4, 12, 12),         # d4b12 (3 bits)
    synth.Shape(1, 3, 1, 128, 1300, 4, 4, 12, 12),        # G = 3
    synth.Shape(2, 8, 2, 128, 777, 4, 8, 10, 12),         # K-d4b10 / V-d8b12 (2 bits on average)
    synth.Shape(1, 16, 2, 128, 1000, 4, 8, 10, 12),
    synth.Shape(2, 8, 2, 128, 800, 8, 8, 12, 8),          # K-d8b12 / V-d8b8 (1.25 bits)
    synth.Shape(1, 8, 2, 128, 1100, 8, 8, 8, 12),         # K-d8b8 / V-d8b12
    synth.Shape(2, 8, 2, 128, 650, 8, 8, 10, 10),         # d8b10 (1.25 bits)
    synth.Shape(1, 2, 2, 128, 1500, 4, 4, 10, 10),        # d4b10, G = 1
    synth.Shape(1, 8, 2, 128, 700, 4, 4, 8, 12),          # 8-bit d4 keys, d4b12 values
    synth.Shape(1, 8, 2, 128, 700, 8, 4, 12, 8),          # d8b12 keys, 8-bit d4 values
    synth.Shape(1, 8, 2, 128, 500, 8, 4, 10, 10),
    # head dim 64 (the second shape of the kernel sweep, App. B.2): d_v = 8 runs as two halves per code
    synth.Shape(2, 8, 2, 64, 777, 8, 8, 12, 12),          # d8b12
    synth.Shape(1, 16, 2, 64, 1300, 8, 8, 12, 12),        # G = 8
    synth.Shape(1, 8, 2, 64, 900, 4, 4, 12, 12),          # d4b12
    synth.Shape(2, 6, 2, 64, 650, 4, 4, 10, 10),          # d4b10, G = 3
    synth.Shape(1, 8, 2, 64, 1000, 4, 8, 10, 12),         # K-d4b10 / V-d8b12
    synth.Shape(1, 8, 2, 64, 800, 8, 8, 12, 8),           # K-d8b12 / V-d8b8
    synth.Shape(1, 4, 1, 64, 4099, 8, 4, 8, 12),          # K-d8b8 / V-d4b12
    synth.Shape(1, 8, 2, 64, 700, 4, 8, 8, 12),           # 8-bit d4 keys, d8b12 values
]


@pytest.mark.parametrize("shape", WIDE, ids=_id)
@pytest.mark.parametrize("splits", [1, 3, 0])
def test_decode_wide(shape, splits):
    x = synth.decode_inputs(shape, seed=shape.N + splits)
    ref = _oracle_decode(shape, x)
    got = gpu_decode(shape, x, num_splits=splits)
    assert_decode_close(*got, *ref, what=f"{_id(shape)} splits={splits}")


def test_decode_wide_ragged_and_degenerate_lengths():
    shape = synth.Shape(4, 8, 2, 128, 900, 8, 8, 12, 12)
    x = synth.decode_inputs(shape, seed=5, n_cap=1024)
    lens = np.array([900, 1, 0, 333])
    got_o, got_l = gpu_decode(shape, x, seq_lens=lens, N=900, num_splits=4)
    keep = [0, 1, 3]
    sub = {k: (v[keep] if k in ("q", "k_idx", "v_idx") else v) for k, v in x.items()}
    ref_o, ref_l = _oracle_decode(shape, sub, lens[keep])
    assert_decode_close(got_o[keep], got_l[keep], ref_o, ref_l, what="wide ragged")
    assert (got_o[2] == 0).all() and np.isneginf(got_l[2]).all()


def test_decode_wide_split_count_invariance():
    shape = synth.Shape(1, 8, 2, 128, 6000, 4, 8, 10, 12)
    x = synth.decode_inputs(shape, seed=9)
    ref = _oracle_decode(shape, x)
    for S in (1, 2, 32, 64, 256):
        assert_decode_close(*gpu_decode(shape, x, num_splits=S), *ref, what=f"wide S={S}")


def test_decode_wide_rejects_the_lookup_table_variant_and_unsupported_shapes():
    shape = synth.Shape(1, 8, 2, 128, 300, 8, 8, 12, 12)
    x = synth.decode_inputs(shape, seed=1)
    with pytest.raises(vb.VecInferError) as e:
        gpu_decode(shape, x, variant=vb.VARIANT_LUT)
    assert e.value.code == vb.EUNSUPPORTED


def test_decode_wide_residual_window():
    """The full-precision window joins the wide-code cache in one softmax (Sec. 4.1)."""
    shape = synth.Shape(2, 8, 2, 128, 1000, 8, 8, 12, 12)
    x = synth.decode_inputs(shape, seed=77)
    x.update(synth.residual_window(shape, seed=78, r_cap=128))
    y = oracle_view(shape, x)
    res_lens = np.array([128, 57])
    ref = oracle.decode_attention_residual(y["q"], y["lam"], y["cb_k"], y["cb_v"], y["k_idx"], y["v_idx"],
                                           y["k_res"], y["v_res"], None, res_lens)
    got = gpu_decode_residual(shape, x, res_lens=res_lens, num_splits=3)
    assert_decode_close(*got, *ref, what="wide residual")


def test_decode_wide_full_size_196k_d8b12():
    """The 8B shape at 196608 tokens with d8b12 keys and values, in the launch configuration the
    benchmark times (auto splits)."""
    shape = synth.LLAMA8B_196K_D8B12
    x = synth.decode_inputs(shape, seed=4)
    ref = _oracle_decode(shape, x)
    got = gpu_decode(shape, x)
    assert_decode_close(*got, *ref, what="d8b12 196k")


# ------------------------------------------------------------------ encode

ENC_WIDE = [
    synth.Shape(2, 2, 2, 128, 200, 8, 8, 12, 12),     # tiled kernel, ragged last tile
    synth.Shape(1, 2, 2, 128, 130, 4, 4, 12, 12),
    synth.Shape(1, 1, 1, 128, 70, 4, 8, 10, 12),
    synth.Shape(1, 2, 2, 128, 90, 8, 4, 10, 10),
    synth.Shape(2, 2, 2, 128, 3, 8, 8, 12, 12),       # per-token kernel
    synth.Shape(1, 2, 2, 128, 16, 4, 4, 10, 12),
    synth.Shape(1, 1, 1, 128, 65, 8, 8, 12, 8),       # one side wide, the other 8-bit
    synth.Shape(2, 2, 2, 64, 200, 8, 8, 12, 12),      # head dim 64
    synth.Shape(1, 2, 1, 64, 130, 4, 4, 10, 12),
    synth.Shape(1, 2, 2, 64, 5, 4, 8, 12, 12),        # per-token kernel
    synth.Shape(1, 1, 1, 64, 70, 8, 4, 12, 8),
]


def _check_encode(shape, e, lam, got_k, got_v, rows, what):
    y = oracle_view(shape, {"cb_k": e["cb_k"], "cb_v": e["cb_v"]})
    ref_k, gap_k = oracle.encode_keys(e["k"], lam, y["cb_k"] if shape.b_k != 8 else e["cb_k"], want_gap=True)
    ref_v, gap_v = oracle.encode_values(e["v"], y["cb_v"] if shape.b_v != 8 else e["cb_v"], want_gap=True)
    uk = oracle.unpack_codes(got_k[:, :, rows], shape.b_k, shape.Mk)
    uv = oracle.unpack_codes(got_v[:, :, rows], shape.b_v, shape.Mv)
    n = assert_indices_match(uk, ref_k, gap_k, what + " keys") + assert_indices_match(uv, ref_v, gap_v, what + " values")
    if n == 0:      # no near-tie: the packed bytes themselves must be the oracle's bit strings
        np.testing.assert_array_equal(got_k[:, :, rows], oracle.pack_codes(ref_k, shape.b_k))
        np.testing.assert_array_equal(got_v[:, :, rows], oracle.pack_codes(ref_v, shape.b_v))


@pytest.mark.parametrize("shape", ENC_WIDE, ids=_id)
def test_encode_wide(shape):
    e = synth.encode_inputs(shape, seed=shape.N, n_outlier=3)
    lam = np.stack([oracle.smoothing_factors(e["k"][:, h]) for h in range(shape.Hkv)]).astype(np.float32)
    got_k, got_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"])
    _check_encode(shape, e, lam, got_k, got_v, slice(0, shape.N), _id(shape))


def test_encode_wide_at_offset_leaves_other_rows_untouched():
    shape = synth.Shape(1, 2, 2, 128, 100, 8, 8, 12, 12)
    e = synth.encode_inputs(shape, seed=8, n_outlier=3)
    lam = synth.lognormal_lambda(synth.rng(9), shape.Hkv, shape.D)
    got_k, got_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"], pos0=37, n_cap=200)
    _check_encode(shape, e, lam, got_k, got_v, slice(37, 137), "offset")
    for got in (got_k, got_v):
        assert (got[:, :, :37] == 0xEE).all() and (got[:, :, 137:] == 0xEE).all()


def test_encode_wide_token_and_tiled_kernels_agree_and_append_equals_encodes():
    """16 tokens go through the per-token kernels, 17 through the tiled ones: same codes for the
    common tokens; vecinfer_append_kv writes what the two encode calls write."""
    shape = synth.Shape(2, 2, 2, 128, 17, 4, 8, 10, 12)
    e = synth.encode_inputs(shape, seed=21, n_outlier=3)
    lam = synth.lognormal_lambda(synth.rng(22), shape.Hkv, shape.D)
    tiled_k, tiled_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"])
    k16, v16 = np.ascontiguousarray(e["k"][:, :, :16]), np.ascontiguousarray(e["v"][:, :, :16])
    tok_k, tok_v = gpu_encode(shape, k=k16, lam=lam, cb_k=e["cb_k"], v=v16, cb_v=e["cb_v"])
    np.testing.assert_array_equal(tok_k, tiled_k[:, :, :16])
    np.testing.assert_array_equal(tok_v, tiled_v[:, :, :16])
    cfg = cfg_of(shape)
    ak = torch.full((2, 2, 40, shape.row_bytes_k), 0xEE, dtype=torch.uint8, device="cuda")
    av = torch.full((2, 2, 40, shape.row_bytes_v), 0xEE, dtype=torch.uint8, device="cuda")
    vb.vecinfer_append_kv(cfg, dev(k16), dev(v16), dev(lam), dev(e["cb_k"]), dev(e["cb_v"]), ak, av, pos0=5)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(ak.cpu().numpy()[:, :, 5:21], tok_k)
    np.testing.assert_array_equal(av.cpu().numpy()[:, :, 5:21], tok_v)
    assert (ak.cpu().numpy()[:, :, :5] == 0xEE).all() and (av.cpu().numpy()[:, :, 21:] == 0xEE).all()


def test_encode_wide_full_size_d8b12_sampled():
    """65536 tokens x 8 KV heads with 12-bit codes on sub-vectors of 8 (the size the cache fill is timed
    at): keys and values, 96 sampled tokens per head against the oracle (Eq. 2 over 4096 centroids)."""
    shape = synth.Shape(1, 8, 8, 128, 65536, 8, 8, 12, 12)
    e = synth.encode_inputs(shape, seed=5, n_outlier=3)
    lam = np.stack([oracle.smoothing_factors(e["k"][:, h]) for h in range(shape.Hkv)]).astype(np.float32)
    got_k, got_v = gpu_encode(shape, k=e["k"], lam=lam, cb_k=e["cb_k"], v=e["v"], cb_v=e["cb_v"])
    rows = np.sort(synth.rng(6).choice(shape.N, size=96, replace=False))
    rows[-1] = shape.N - 1
    ref_k, gap_k = oracle.encode_keys(e["k"][:, :, rows], lam, e["cb_k"][:, None], want_gap=True)
    ref_v, gap_v = oracle.encode_values(e["v"][:, :, rows], e["cb_v"][:, None], want_gap=True)
    assert_indices_match(oracle.unpack_codes(got_k[:, :, rows], 12, shape.Mk), ref_k, gap_k, "d8b12 keys, 65536 tokens")
    assert_indices_match(oracle.unpack_codes(got_v[:, :, rows], 12, shape.Mv), ref_v, gap_v, "d8b12 values, 65536 tokens")


def test_encode_wide_planted_codes_and_ties():
    """Vectors built from centroids come back as those codes; a duplicated centroid resolves to
    its lowest index (Eq. 2 with the lowest-index rule)."""
    shape = synth.Shape(1, 1, 1, 128, 150, 8, 8, 12, 12)
    g = synth.rng(31)
    cb = synth.shared_codebooks(g, 1, 12, 8)
    cb[0, 3000] = cb[0, 17]
    pick = g.integers(0, 4096, size=(1, 1, shape.N, 16))
    pick[0, 0, :, 3] = 3000
    v = cb[0][pick[0, 0]].reshape(1, 1, shape.N, 128)
    (got_v,) = gpu_encode(shape, v=v, cb_v=cb)
    want = np.where(pick == 3000, 17, pick)
    first = {}                                    # other accidental duplicates: lowest index of equal rows
    for c in range(4096):
        first.setdefault(cb[0, c].tobytes(), c)
    want = np.vectorize(lambda c: first[cb[0, c].tobytes()])(want)
    np.testing.assert_array_equal(oracle.unpack_codes(got_v, 12, 16), want)


# ------------------------------------------------------------------ whole step

def test_decode_step_wide_equals_append_then_attend_and_the_oracle():
    shape = synth.Shape(2, 8, 2, 128, 1200, 8, 8, 12, 12)
    x = synth.decode_inputs(shape, seed=51, n_cap=1300)
    g = synth.rng(52)
    k_new, _ = synth.keys_with_outlier_channels(g, shape.B, shape.Hkv, 1, shape.D, 3)
    v_new = synth.values(g, shape.B, shape.Hkv, 1, shape.D)
    cfg = cfg_of(shape)
    lens = np.array([1200, 431])
    t = {k: dev(v) for k, v in x.items()}
    ws = vb.new_workspace(cfg, shape.B, shape.N)
    out = torch.empty((shape.B, shape.Hq, shape.D), dtype=torch.float16, device="cuda")
    lse = torch.empty((shape.B, shape.Hq), dtype=torch.float32, device="cuda")
    vb.vecinfer_decode_step(cfg, t["q"], dev(k_new), dev(v_new), t["lam"], t["cb_k"], t["cb_v"], t["k_idx"],
                            t["v_idx"], ws, out, lse=lse, seq_lens=torch.as_tensor(lens, dtype=torch.int32).cuda(),
                            N=shape.N)
    torch.cuda.synchronize()
    k_idx, v_idx = t["k_idx"].cpu().numpy(), t["v_idx"].cpu().numpy()
    # the appended rows are the oracle's codes of the new token; every other row is untouched
    y = oracle_view(shape, {"cb_k": x["cb_k"], "cb_v": x["cb_v"]})
    ref_k, gap_k = oracle.encode_keys(k_new, x["lam"], y["cb_k"], want_gap=True)
    ref_v, gap_v = oracle.encode_values(v_new, y["cb_v"], want_gap=True)
    for b in range(shape.B):
        row = lens[b] - 1
        assert_indices_match(oracle.unpack_codes(k_idx[b, :, row], 12, 16), ref_k[b, :, 0], gap_k[b, :, 0], "step keys")
        assert_indices_match(oracle.unpack_codes(v_idx[b, :, row], 12, 16), ref_v[b, :, 0], gap_v[b, :, 0], "step values")
        keep = np.ones(k_idx.shape[2], dtype=bool)
        keep[row] = False
        np.testing.assert_array_equal(k_idx[b][:, keep], x["k_idx"][b][:, keep])
        np.testing.assert_array_equal(v_idx[b][:, keep], x["v_idx"][b][:, keep])
    ref = _oracle_decode(shape, dict(x, k_idx=k_idx, v_idx=v_idx), lens)
    assert_decode_close(out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64), *ref,
                        what="wide step")


# ------------------------------------------------------------------ K-Means step on a shared codebook

@pytest.mark.parametrize("kind", ["keys", "values"])
@pytest.mark.parametrize("shape", [synth.Shape(2, 2, 2, 128, 500, 8, 8, 12, 12), synth.Shape(1, 2, 2, 128, 330, 4, 8, 10, 12)],
                         ids=_id)
def test_kmeans_step_wide(shape, kind):
    """One Lloyd iteration of a KV head's one codebook over the pooled sub-vectors (Sec. 2.2):
    assignment against the oracle's Eq. 2, counts exact, centroids against the oracle's means for
    the GPU's own assignment (fp32 atomic sums, fp16 result), empty clusters bit for bit."""
    e = synth.encode_inputs(shape, seed=shape.N + 7, n_outlier=3)
    keys = kind == "keys"
    if keys:
        lam = np.stack([oracle.smoothing_factors(e["k"][:, h]) for h in range(shape.Hkv)]).astype(np.float32)
        x, cb, bits, M = e["k"], e["cb_k"], shape.b_k, shape.Mk
    else:
        lam, x, cb, bits, M = None, e["v"], e["cb_v"], shape.b_v, shape.Mv
    cfg = cfg_of(shape)
    B, Hkv, T, D = x.shape
    cb_out = torch.full(cb.shape, float("nan"), dtype=torch.float16, device="cuda")
    codes = torch.full((B, Hkv, T, M * bits // 8), 0xEE, dtype=torch.uint8, device="cuda")
    counts = torch.full(cb.shape[:-1], -1, dtype=torch.int32, device="cuda")
    ws = vb.new_kmeans_workspace(cfg, keys)
    vb.vecinfer_kmeans_step(cfg, dev(x), None if lam is None else dev(lam), dev(cb), cb_out, codes, ws, counts=counts)
    torch.cuda.synchronize()
    cb_out, counts = cb_out.cpu().numpy(), counts.cpu().numpy()
    got_idx = oracle.unpack_codes(codes.cpu().numpy(), bits, M)
    ocb = cb[:, None]
    ref_idx, gap = (oracle.encode_keys(x, lam, ocb, want_gap=True) if keys else
                    oracle.encode_values(x, ocb, want_gap=True))
    assert_indices_match(got_idx, ref_idx, gap, f"kmeans wide {kind}: assignment")
    for g in range(Hkv):
        rows = x[:, g].reshape(B * T, D).astype(np.float64)
        if keys:
            rows = oracle.transform_keys(rows, lam[g])
        ref_cb, ref_counts = oracle.kmeans_update(rows, got_idx[:, g].reshape(B * T, M), ocb[g])
        np.testing.assert_array_equal(counts[g], ref_counts[0])
        assert ref_counts.sum() == B * T * M and (ref_counts == 0).any()
        np.testing.assert_allclose(cb_out[g].astype(np.float64), ref_cb[0], rtol=1.5e-3, atol=1e-6)
        empty = ref_counts[0] == 0
        np.testing.assert_array_equal(cb_out[g][empty], cb[g][empty])


STEP_WIDE = [
    synth.Shape(2, 8, 2, 128, 1200, 8, 8, 12, 12),
    synth.Shape(1, 8, 2, 128, 2100, 4, 8, 10, 12),
    synth.Shape(2, 4, 1, 128, 700, 4, 4, 12, 12),
    synth.Shape(1, 16, 2, 128, 900, 8, 8, 10, 10),       # G = 8
    # G = 8 with small shared tables: with one split the wavefronts' partials (32 KB) reach past the
    # tables into the new token's scratch, which must have been read by then
    synth.Shape(1, 16, 2, 128, 900, 4, 4, 10, 10),
    synth.Shape(1, 16, 2, 128, 900, 4, 8, 10, 10),
    synth.Shape(2, 12, 2, 128, 333, 4, 4, 10, 10),       # G = 6
    synth.Shape(2, 8, 2, 128, 800, 8, 8, 12, 8),         # keys wide, values 8-bit
    synth.Shape(1, 6, 2, 128, 650, 4, 8, 8, 12),         # keys 8-bit, values wide, G = 3
    synth.Shape(1, 8, 2, 128, 1, 8, 8, 12, 12),          # the new token is the only one
    synth.Shape(2, 8, 2, 64, 1200, 8, 8, 12, 12),        # head dim 64
    synth.Shape(1, 8, 2, 64, 900, 4, 8, 10, 12),
    synth.Shape(1, 16, 2, 64, 700, 4, 4, 12, 10),        # G = 8
    synth.Shape(2, 4, 2, 64, 650, 8, 4, 12, 8),
    synth.Shape(1, 6, 2, 64, 500, 4, 8, 8, 12),
]


@pytest.mark.parametrize("shape", STEP_WIDE, ids=_id)
@pytest.mark.parametrize("splits", [1, 5, 64, 0])
def test_decode_step_wide_fused_equals_append_then_attend(shape, splits):
    """The whole step with wide codes encodes the new token inside the attention launch: the
    packed rows must be bit-identical to what vecinfer_append_kv writes, and the output equal to
    vecinfer_decode_attention on the result (and to the oracle)."""
    x = synth.decode_inputs(shape, seed=shape.N + 5, n_cap=shape.N + 4)   # (+ 4: per-sequence slices of 12-byte rows stay 16-byte aligned)
    g = synth.rng(shape.N + 6)
    k_new, _ = synth.keys_with_outlier_channels(g, shape.B, shape.Hkv, 1, shape.D, 3)
    v_new = synth.values(g, shape.B, shape.Hkv, 1, shape.D)
    lens = np.array([shape.N] + [max(1, shape.N // 3)] * (shape.B - 1))
    sl = torch.as_tensor(lens, dtype=torch.int32).cuda()
    cfg = cfg_of(shape)
    t = {k: dev(v) for k, v in x.items()}
    ws = vb.new_workspace(cfg, shape.B, shape.N, splits)
    out = torch.full((shape.B, shape.Hq, shape.D), float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full((shape.B, shape.Hq), float("nan"), dtype=torch.float32, device="cuda")
    vb.vecinfer_decode_step(cfg, t["q"], dev(k_new), dev(v_new), t["lam"], t["cb_k"], t["cb_v"], t["k_idx"],
                            t["v_idx"], ws, out, lse=lse, seq_lens=sl, N=shape.N, num_splits=splits)
    torch.cuda.synchronize()
    # the same append by the append kernels, one sequence at a time (each has its own position)
    k2, v2 = dev(x["k_idx"]), dev(x["v_idx"])
    for b in range(shape.B):
        vb.vecinfer_append_kv(cfg, dev(k_new[b:b + 1]), dev(v_new[b:b + 1]), t["lam"], t["cb_k"], t["cb_v"],
                              k2[b:b + 1], v2[b:b + 1], pos0=int(lens[b]) - 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t["k_idx"].cpu().numpy(), k2.cpu().numpy())
    np.testing.assert_array_equal(t["v_idx"].cpu().numpy(), v2.cpu().numpy())
    got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
    ref_gpu = gpu_decode(shape, dict(x, k_idx=k2, v_idx=v2), seq_lens=lens, N=shape.N, num_splits=splits)
    assert_decode_close(*got, *ref_gpu, what="fused wide step vs append + attend")
    ref = _oracle_decode(shape, dict(x, k_idx=k2.cpu().numpy(), v_idx=v2.cpu().numpy()), lens)
    assert_decode_close(*got, *ref, what="fused wide step vs oracle")
