"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests re-types an oracle formula and compares it with itself: each
one checks the oracle against a closed form, a hand-worked value, an invariant,
a textbook special case, a library routine (scipy / torch, float64) or a brute
force written in a different way (vectorised numpy instead of C loops).
"""
import os

import numpy as np
import pytest
import scipy.linalg
import scipy.spatial.distance
import scipy.special
import torch

from paper_2510_06175_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _blocks(path):
    blocks, cur = [], []
    for line in open(path):
        s = line.strip()
        if s.startswith("#"):
            continue
        if not s:
            if cur:
                blocks.append(np.array(cur, dtype=np.float64))
                cur = []
            continue
        cur.append([float(t) for t in s.split()])
    if cur:
        blocks.append(np.array(cur, dtype=np.float64))
    return blocks


# --------------------------------------------------------------------------- Hadamard (Eq. 5)

def test_hadamard_h4_golden(oracle):
    (h4x2,) = _blocks(os.path.join(GOLDEN, "hadamard_h4.txt"))
    np.testing.assert_allclose(oracle.hadamard(4) * 2.0, h4x2, rtol=0, atol=1e-15)


def test_hadamard_h2_closed_form(oracle):
    r = 1.0 / np.sqrt(2.0)
    np.testing.assert_allclose(oracle.hadamard(2), [[r, r], [r, -r]], rtol=0, atol=1e-16)
    np.testing.assert_array_equal(oracle.hadamard(1), [[1.0]])


@pytest.mark.parametrize("D", [2, 8, 64, 128])
def test_hadamard_properties(oracle, D):
    H = oracle.hadamard(D)
    # orthonormal (Sec. 3.2: H H^T = I); the un-normalised butterfly matrix gives D * I
    np.testing.assert_allclose(H @ H.T, np.eye(D), atol=1e-13)
    U = H * np.sqrt(D)
    np.testing.assert_allclose(U @ U.T, D * np.eye(D), atol=1e-10)
    # entries are +-1/sqrt(D) (proof of Lemma 1) with the Sylvester sign (-1)^popcount(i & j)
    i, j = np.meshgrid(np.arange(D), np.arange(D), indexing="ij")
    sign = 1.0 - 2.0 * (np.array([[bin(a & b).count("1") & 1 for b in range(D)] for a in range(D)]))
    np.testing.assert_allclose(H, sign / np.sqrt(D), atol=1e-15)
    # library construction of the same (Sylvester) matrix
    np.testing.assert_allclose(H, scipy.linalg.hadamard(D) / np.sqrt(D), atol=1e-15)
    np.testing.assert_array_equal(H, H.T)
    # first unit vector maps to the constant row; the transform is an involution and an isometry
    np.testing.assert_allclose(np.eye(D)[0] @ H, np.full(D, 1 / np.sqrt(D)), atol=1e-15)
    x = synth.rng(D).standard_normal(D)
    np.testing.assert_allclose((x @ H) @ H, x, atol=1e-13)
    np.testing.assert_allclose(np.linalg.norm(x @ H), np.linalg.norm(x), rtol=1e-13)


def test_hadamard_rejects_non_power_of_two(oracle):
    with pytest.raises(ValueError):
        oracle.hadamard(96)


# --------------------------------------------------------------------------- smoothing (Eq. 3, Eq. 4)

def test_smoothing_factors_golden(oracle):
    K, lam = _blocks(os.path.join(GOLDEN, "smoothing_example.txt"))
    np.testing.assert_array_equal(oracle.smoothing_factors(K), lam[0])


def test_transform_direction_on_unit_vectors(oracle):
    """Keys are divided by lambda and queries multiplied (Eq. 3), each then times H (Eq. 6)."""
    D = 16
    lam = np.linspace(0.5, 4.0, D)
    H = scipy.linalg.hadamard(D) / np.sqrt(D)
    for i in (0, 3, 15):
        e = np.zeros(D)
        e[i] = 1.0
        np.testing.assert_allclose(oracle.transform_keys(e[None, :], lam)[0], H[i] / lam[i], atol=1e-15)
        np.testing.assert_allclose(oracle.transform_query(e, lam), H[i] * lam[i], atol=1e-15)


def test_transform_matches_library_matmul(oracle):
    g = synth.rng(11)
    D = 128
    K = g.standard_normal((37, D))
    lam = np.exp(0.5 * g.standard_normal(D))
    H = scipy.linalg.hadamard(D) / np.sqrt(D)
    np.testing.assert_allclose(oracle.transform_keys(K, lam), (K / lam) @ H, atol=1e-12)
    np.testing.assert_allclose(oracle.transform_query(K[0], lam), (K[0] * lam) @ H, atol=1e-12)


def test_score_invariance_under_dual_transform(oracle):
    """Eq. 7: (q diag(lam) H)(K diag(lam)^-1 H)^T = q K^T for any lam > 0."""
    g = synth.rng(7)
    D = 128
    K = g.standard_normal((64, D)) * np.where(g.random(D) < 0.05, 20.0, 1.0)
    q = g.standard_normal(D)
    lam = np.exp(0.5 * g.standard_normal(D))
    qt = oracle.transform_query(q, lam)
    Kt = oracle.transform_keys(K, lam)
    np.testing.assert_allclose(Kt @ qt, K @ q, rtol=1e-11, atol=1e-11)
    # with Eq. 4's lambda as well
    lam4 = oracle.smoothing_factors(K)
    np.testing.assert_allclose(oracle.transform_keys(K, lam4) @ oracle.transform_query(q, lam4),
                               K @ q, rtol=1e-11, atol=1e-11)


def test_lemma1_row_energy_and_outlier_suppression(oracle):
    """Lemma 1: each transformed entry has variance (1/D) sum_l K_il^2; as H is orthonormal the
    row's mean square equals exactly that.  Smooth + Hadamard flattens the outlier channels."""
    e = synth.encode_inputs(synth.TINY, seed=1, n_outlier=4)
    K = e["k"][0, 0].astype(np.float64)
    lam = oracle.smoothing_factors(K)
    Kt = oracle.transform_keys(K, lam)
    np.testing.assert_allclose((Kt ** 2).mean(axis=1), ((K / lam) ** 2).sum(axis=1) / K.shape[1], rtol=1e-12)
    spread = lambda X: np.abs(X).max(axis=0).max() / np.abs(X).max(axis=0).min()
    assert spread(K) > 10.0 and spread(Kt) < 2.5


# --------------------------------------------------------------------------- VQ encode (Eq. 2, Eq. 8)

@pytest.mark.parametrize("d", [2, 4, 8])
def test_vq_encode_vs_cdist_brute_force(oracle, d):
    g = synth.rng(100 + d)
    D, N, C = 32, 50, 256
    M = D // d
    X = g.standard_normal((N, D))
    cb = g.standard_normal((M, C, d))
    idx = oracle.vq_encode(X, cb)
    assert idx.dtype == np.uint8 and idx.shape == (N, M)
    for m in range(M):
        dist = scipy.spatial.distance.cdist(X[:, m * d:(m + 1) * d], cb[m], metric="sqeuclidean")
        np.testing.assert_array_equal(idx[:, m], dist.argmin(axis=1))


def test_vq_encode_ties_take_lowest_index_and_gap_is_zero(oracle):
    g = synth.rng(5)
    cb = g.standard_normal((2, 256, 4))
    cb[:, 200] = cb[:, 17]          # exact duplicates
    X = np.concatenate([cb[0, 17], cb[1, 200]])[None, :]
    idx, gap = oracle.vq_encode(X, cb, want_gap=True)
    np.testing.assert_array_equal(idx, [[17, 17]])
    np.testing.assert_array_equal(gap, [[0.0, 0.0]])


def test_vq_encode_gap_is_relative_distance_gap(oracle):
    cb = np.zeros((1, 256, 2))
    cb[0, :, 0] = 10.0 + np.arange(256)
    cb[0, 3] = [1.0, 0.0]           # distance^2 to origin 1
    cb[0, 9] = [0.0, 2.0]           # distance^2 to origin 4
    idx, gap = oracle.vq_encode(np.zeros((1, 2)), cb, want_gap=True)
    assert idx[0, 0] == 3 and gap[0, 0] == pytest.approx(3.0)


def test_vq_encode_centroid_in_index_out_and_permutation(oracle):
    g = synth.rng(6)
    M, C, d = 8, 256, 4
    cb = g.standard_normal((M, C, d))
    want = g.integers(0, C, size=(40, M), dtype=np.uint8)
    X = oracle.vq_dequantize(want, cb)
    np.testing.assert_array_equal(X[3, 4:8], cb[1, want[3, 1]])     # dequantize = centroid lookup
    np.testing.assert_array_equal(oracle.vq_encode(X, cb), want)
    # permuting every codebook permutes the indices the same way
    perm = g.permutation(C)
    inv = np.argsort(perm)
    Y = g.standard_normal((40, M * d))
    np.testing.assert_array_equal(oracle.vq_encode(Y, cb[:, perm]), inv[oracle.vq_encode(Y, cb)])


def test_code_and_codebook_sizes():
    """Sec. 2.2: (d_h/d)(b/8) index bytes per vector and 2^b d 2 codebook bytes."""
    s = synth.LLAMA8B_196K
    assert s.Mk == 32 and s.Mk * 8 // 8 == 32 and synth.NUM_CENTROIDS * s.d_k * 2 == 2048
    s2 = synth.LLAMA8B_196K_B4D2
    assert s2.Mk == 64 and synth.NUM_CENTROIDS * s2.d_k * 2 == 1024
    assert s.index_bytes() == 100663296 and s2.index_bytes() == 201326592


def test_encode_keys_recovers_planted_codes(oracle):
    """K = (concatenated centroids) H^T diag(lam) must encode to exactly the planted codes,
    for per-head codebooks and smoothing factors (Alg. 1 steps 2-3)."""
    g = synth.rng(8)
    B, Hkv, T, D, d = 2, 3, 9, 128, 4
    M = D // d
    cb = synth.codebooks(g, Hkv, M, d)
    lam = synth.lognormal_lambda(g, Hkv, D)
    want = g.integers(0, 256, size=(B, Hkv, T, M), dtype=np.uint8)
    H = scipy.linalg.hadamard(D) / np.sqrt(D)
    K = np.empty((B, Hkv, T, D))
    for b in range(B):
        for h in range(Hkv):
            Khat = cb[h].astype(np.float64)[np.arange(M)[None, :], want[b, h]].reshape(T, D)
            K[b, h] = (Khat @ H.T) * lam[h].astype(np.float64)
    got = oracle.encode_keys(K, lam, cb)
    # distinct fp16 centroids ~N(0,1) are separated by far more than float64 rounding
    np.testing.assert_array_equal(got, want)
    # values: no transform at all
    V = np.stack([[cb[h].astype(np.float64)[np.arange(M)[None, :], want[b, h]].reshape(T, D)
                   for h in range(Hkv)] for b in range(B)])
    np.testing.assert_array_equal(oracle.encode_values(V, cb), want)


def test_encode_keys_vs_numpy_pipeline(oracle):
    e = synth.encode_inputs(synth.Shape(B=1, Hq=2, Hkv=2, D=128, N=33, d_k=4, d_v=2), seed=3, n_outlier=3)
    lam = np.stack([oracle.smoothing_factors(e["k"][:, h]) for h in range(2)]).astype(np.float32)
    H = scipy.linalg.hadamard(128) / np.sqrt(128)
    got, gap = oracle.encode_keys(e["k"], lam, e["cb_k"], want_gap=True)
    gotv = oracle.encode_values(e["v"], e["cb_v"])
    assert got.shape == (1, 2, 33, 32) and gotv.shape == (1, 2, 33, 64)
    for h in range(2):
        Kt = (e["k"][0, h].astype(np.float64) / lam[h].astype(np.float64)) @ H
        for m in range(32):
            dist = scipy.spatial.distance.cdist(Kt[:, 4 * m:4 * m + 4], e["cb_k"][h, m].astype(np.float64),
                                                "sqeuclidean")
            ok = (dist.argmin(axis=1) == got[0, h, :, m]) | (gap[0, h, :, m] < 1e-9)
            assert ok.all()
        V = e["v"][0, h].astype(np.float64)
        for m in range(64):
            dist = scipy.spatial.distance.cdist(V[:, 2 * m:2 * m + 2], e["cb_v"][h, m].astype(np.float64),
                                                "sqeuclidean")
            np.testing.assert_array_equal(dist.argmin(axis=1), gotv[0, h, :, m])


# --------------------------------------------------------------------------- VQ attention (Eq. 10, Alg. 1)

def _dequant_np(idx, cb):
    """idx [N, M], cb [M, C, d] -> [N, M*d] by numpy fancy indexing (not the oracle's loop)."""
    M = cb.shape[0]
    return cb.astype(np.float64)[np.arange(M)[None, :], idx].reshape(idx.shape[0], -1)


def _small_decode_case(seed, B=2, Hq=4, Hkv=2, D=64, N=75, d_k=4, d_v=2):
    return synth.Shape(B, Hq, Hkv, D, N, d_k, d_v), synth.decode_inputs(
        synth.Shape(B, Hq, Hkv, D, N, d_k, d_v), seed)


def test_decode_matches_torch_sdpa_on_dequantized_cache(oracle):
    """Eq. 10 is textbook attention (Eq. 1) on the dequantized cache with the transformed query."""
    s, x = _small_decode_case(21)
    seq = np.array([75, 41])
    out, lse = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"], seq)
    H = scipy.linalg.hadamard(s.D) / np.sqrt(s.D)
    for b in range(s.B):
        n = seq[b]
        Kh = np.stack([_dequant_np(x["k_idx"][b, g, :n], x["cb_k"][g]) for g in range(s.Hkv)])
        Vh = np.stack([_dequant_np(x["v_idx"][b, g, :n], x["cb_v"][g]) for g in range(s.Hkv)])
        lam_q = np.repeat(x["lam"].astype(np.float64), s.G, axis=0)           # head h -> KV head h // G
        qt = (x["q"][b].astype(np.float64) * lam_q) @ H
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(qt)[None, :, None, :],
            torch.from_numpy(Kh).repeat_interleave(s.G, dim=0)[None],
            torch.from_numpy(Vh).repeat_interleave(s.G, dim=0)[None])[0, :, 0].numpy()
        np.testing.assert_allclose(out[b], ref, rtol=1e-11, atol=1e-13)
        scores = np.einsum("hd,hnd->hn", qt, np.repeat(Kh, s.G, axis=0)) / np.sqrt(s.D)
        np.testing.assert_allclose(lse[b], scipy.special.logsumexp(scores, axis=1), rtol=1e-12)


def test_decode_zero_query_gives_mean_of_values_and_log_n(oracle):
    s, x = _small_decode_case(22, B=1, Hq=2, Hkv=1, N=50)
    x["q"][:] = 0
    out, lse = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    Vh = _dequant_np(x["v_idx"][0, 0], x["cb_v"][0])
    np.testing.assert_allclose(out[0, 0], Vh.mean(axis=0), atol=1e-14)
    np.testing.assert_allclose(out[0, 1], Vh.mean(axis=0), atol=1e-14)
    np.testing.assert_allclose(lse, np.log(50.0), rtol=1e-14)


def test_decode_single_token(oracle):
    s, x = _small_decode_case(23, B=1, Hq=2, Hkv=2, N=1)
    out, lse = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    H = scipy.linalg.hadamard(s.D) / np.sqrt(s.D)
    for h in range(2):
        np.testing.assert_allclose(out[0, h], _dequant_np(x["v_idx"][0, h], x["cb_v"][h])[0], atol=1e-15)
        qt = (x["q"][0, h].astype(np.float64) * x["lam"][h].astype(np.float64)) @ H
        s0 = qt @ _dequant_np(x["k_idx"][0, h], x["cb_k"][h])[0] / np.sqrt(s.D)
        np.testing.assert_allclose(lse[0, h], s0, rtol=1e-12)


def test_decode_output_is_convex_combination(oracle):
    s, x = _small_decode_case(24)
    out, _ = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    for b in range(s.B):
        for h in range(s.Hq):
            Vh = _dequant_np(x["v_idx"][b, h // s.G], x["cb_v"][h // s.G])
            assert (out[b, h] <= Vh.max(axis=0) + 1e-12).all() and (out[b, h] >= Vh.min(axis=0) - 1e-12).all()


@pytest.mark.parametrize("tile", [1, 7, 64, 1000])
def test_alg1_lookup_online_softmax_equals_eq10(oracle, tile):
    """LUT-sum score = explicit dot, and the tiled online softmax = plain softmax (Alg. 1 vs Eq. 10)."""
    s, x = _small_decode_case(25)
    seq = np.array([75, 13])
    a = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"], seq)
    b = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"], seq,
                                path="alg1", tile=tile)
    np.testing.assert_allclose(b[0], a[0], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(b[1], a[1], rtol=1e-12)


@pytest.mark.parametrize("cuts", [[0, 75], [0, 1, 75], [0, 20, 21, 50, 75]])
def test_split_merge_equals_whole(oracle, cuts):
    s, x = _small_decode_case(26, B=1, Hq=2, Hkv=1)
    whole, L = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    parts_o, parts_L = [], []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        o, l = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"],
                                       x["k_idx"][:, :, lo:hi], x["v_idx"][:, :, lo:hi])
        parts_o.append(o[0])
        parts_L.append(l[0])
    for h in range(2):
        o, l = oracle.merge_splits(np.stack([p[h] for p in parts_o]), np.array([p[h] for p in parts_L]))
        np.testing.assert_allclose(o, whole[0, h], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(l, L[0, h], rtol=1e-12)
    # merge identity on two scalars: L = log(e^{L1} + e^{L2})
    _, l = oracle.merge_splits(np.zeros((2, 4)), np.array([0.3, -1.2]))
    assert l == pytest.approx(np.log(np.exp(0.3) + np.exp(-1.2)), rel=1e-14)


def test_softmax_shift_invariance(oracle):
    """Adding one vector u to every centroid of one key sub-space adds q~_m . u / sqrt(D) to every
    score: the output is unchanged and L moves by exactly that amount."""
    s, x = _small_decode_case(27, B=1, Hq=2, Hkv=1)
    base_o, base_L = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    cb2 = x["cb_k"].astype(np.float64).copy()
    u = np.array([0.5, -1.0, 2.0, 0.25])
    cb2[0, 5] += u
    o2, L2 = oracle.decode_attention(x["q"], x["lam"], cb2, x["cb_v"], x["k_idx"], x["v_idx"])
    np.testing.assert_allclose(o2, base_o, rtol=1e-10, atol=1e-13)
    for h in range(2):
        qt = oracle.transform_query(x["q"][0, h], x["lam"][0])
        np.testing.assert_allclose(L2[0, h] - base_L[0, h], qt[20:24] @ u / np.sqrt(s.D), rtol=1e-9)


# --------------------------------------------------------------------------- residual window (Sec. 4.1)

def _residual_case(seed, B=2, Hq=4, Hkv=2, D=64, N=75, R=9):
    s, x = _small_decode_case(seed, B=B, Hq=Hq, Hkv=Hkv, D=D, N=N)
    g = synth.rng(seed + 1000)
    x["k_res"] = (g.standard_normal((B, Hkv, R, D)) * np.where(g.random(D) < 0.1, 8.0, 1.0)).astype(np.float16)
    x["v_res"] = g.standard_normal((B, Hkv, R, D)).astype(np.float16)
    return s, x


def test_residual_window_matches_sdpa_on_concatenated_cache(oracle):
    """The window's raw-query x raw-key scores equal transformed-query x transformed-key scores
    (Eq. 7), so the result is textbook attention of q~ over [K^ ; k~_res] and [V^ ; v_res]."""
    s, x = _residual_case(41)
    seq, res = np.array([75, 40]), np.array([9, 4])
    out, lse = oracle.decode_attention_residual(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"],
                                                x["k_res"], x["v_res"], seq, res)
    H = scipy.linalg.hadamard(s.D) / np.sqrt(s.D)
    for b in range(s.B):
        n, r = seq[b], res[b]
        K, V = [], []
        for g in range(s.Hkv):
            kt_res = (x["k_res"][b, g, :r].astype(np.float64) / x["lam"][g].astype(np.float64)) @ H
            K.append(np.concatenate([_dequant_np(x["k_idx"][b, g, :n], x["cb_k"][g]), kt_res]))
            V.append(np.concatenate([_dequant_np(x["v_idx"][b, g, :n], x["cb_v"][g]),
                                     x["v_res"][b, g, :r].astype(np.float64)]))
        lam_q = np.repeat(x["lam"].astype(np.float64), s.G, axis=0)
        qt = (x["q"][b].astype(np.float64) * lam_q) @ H
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(qt)[None, :, None, :],
            torch.from_numpy(np.stack(K)).repeat_interleave(s.G, dim=0)[None],
            torch.from_numpy(np.stack(V)).repeat_interleave(s.G, dim=0)[None])[0, :, 0].numpy()
        np.testing.assert_allclose(out[b], ref, rtol=1e-10, atol=1e-12)
        scores = np.einsum("hd,hnd->hn", qt, np.repeat(np.stack(K), s.G, axis=0)) / np.sqrt(s.D)
        np.testing.assert_allclose(lse[b], scipy.special.logsumexp(scores, axis=1), rtol=1e-11)


def test_residual_window_special_cases(oracle):
    s, x = _residual_case(42, B=1, Hq=2, Hkv=1, N=30, R=5)
    base = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    # an empty window changes nothing
    o0, l0 = oracle.decode_attention_residual(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"],
                                              x["k_res"], x["v_res"], res_lens=np.array([0]))
    np.testing.assert_array_equal(o0, base[0])
    np.testing.assert_array_equal(l0, base[1])
    # no quantized token at all: plain attention (Eq. 1) of the raw query over the window
    o1, l1 = oracle.decode_attention_residual(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"],
                                              x["k_res"], x["v_res"], seq_lens=np.array([0]))
    q = x["q"][0].astype(np.float64)
    K = x["k_res"][0, 0].astype(np.float64)
    V = x["v_res"][0, 0].astype(np.float64)
    sc = q @ K.T / np.sqrt(s.D)
    np.testing.assert_allclose(o1[0], scipy.special.softmax(sc, axis=1) @ V, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(l1[0], scipy.special.logsumexp(sc, axis=1), rtol=1e-12)
    # window and quantized part attended separately, then merged by log-sum-exp = joint result
    joint, L = oracle.decode_attention_residual(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"],
                                                x["k_res"], x["v_res"])
    for h in range(2):
        o, l = oracle.merge_splits(np.stack([base[0][0, h], o1[0, h]]), np.array([base[1][0, h], l1[0, h]]))
        np.testing.assert_allclose(o, joint[0, h], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(l, L[0, h], rtol=1e-12)
    with pytest.raises(ValueError):
        oracle.decode_attention_residual(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"],
                                         x["k_res"], x["v_res"], seq_lens=np.array([0]), res_lens=np.array([0]))


# --------------------------------------------------------------------------- K-Means step (Sec. 2.2, 4.1)

def test_kmeans_update_matches_scipy_lloyd_iteration(oracle):
    """One sub-space, 256 centroids: scipy's kmeans2 with a given start and one iteration does
    exactly assignment (Eq. 2) + mean update; an empty cluster keeps its centroid there too."""
    import warnings
    from scipy.cluster.vq import kmeans2
    g = synth.rng(51)
    for d in (2, 4, 8):
        X = g.standard_normal((3000, d))
        init = g.standard_normal((256, d)) * 1.5
        init[7] = 50.0                                   # far away: stays empty
        idx = oracle.vq_encode(X, init[None])
        new, counts = oracle.kmeans_update(X, idx, init[None])
        with warnings.catch_warnings():
            warnings.simplefilter("ignore")
            ref, label = kmeans2(X, init.copy(), iter=1, minit="matrix")
        np.testing.assert_array_equal(idx[:, 0], label)
        np.testing.assert_allclose(new[0], ref, rtol=1e-12, atol=1e-14)
        np.testing.assert_array_equal(counts[0], np.bincount(label, minlength=256))
        assert counts[0, 7] == 0 and (new[0, 7] == 50.0).all()


def test_kmeans_update_is_the_mean_per_sub_space_and_code(oracle):
    g = synth.rng(52)
    D, d, N = 16, 4, 500
    X = g.standard_normal((N, D))
    cb = g.standard_normal((D // d, 256, d))
    idx = g.integers(0, 5, size=(N, D // d)).astype(np.uint8)          # any assignment, not only the nearest
    new, counts = oracle.kmeans_update(X, idx, cb)
    for m in range(D // d):
        for c in range(256):
            sel = idx[:, m] == c
            assert counts[m, c] == sel.sum()
            want = X[sel, m * d:(m + 1) * d].mean(axis=0) if sel.any() else cb[m, c]
            np.testing.assert_allclose(new[m, c], want, rtol=1e-12, atol=1e-14)


def test_kmeans_step_never_increases_the_quantization_error(oracle):
    """Lloyd's monotonicity over the batched entry (keys: on the transformed keys), and a fixed
    point: centroids that already are the means of their clusters do not move."""
    g = synth.rng(53)
    B, Hkv, T, D, d = 2, 2, 700, 64, 4
    k, _ = synth.keys_with_outlier_channels(g, B, Hkv, T, D, 2)
    lam = np.stack([oracle.smoothing_factors(k[:, h]) for h in range(Hkv)])
    cb = synth.codebooks(g, Hkv, D // d, d).astype(np.float64)

    def error(cbx):
        tot = 0.0
        idx = oracle.encode_keys(k, lam, cbx)
        for h in range(Hkv):
            rows = oracle.transform_keys(k[:, h].reshape(B * T, D).astype(np.float64), lam[h])
            tot += ((rows - oracle.vq_dequantize(idx[:, h].reshape(B * T, -1), cbx[h])) ** 2).sum()
        return tot

    errs = [error(cb)]
    for _ in range(4):
        cb, counts, _ = oracle.kmeans_step(k, lam, cb)
        assert counts.sum() == Hkv * (D // d) * B * T
        errs.append(error(cb))
    assert all(b <= a * (1 + 1e-12) for a, b in zip(errs, errs[1:])) and errs[-1] < 0.8 * errs[0]
    for _ in range(60):                                   # run to the fixed point
        nxt, _, _ = oracle.kmeans_step(k, lam, cb)
        if np.array_equal(nxt, cb):
            break
        cb = nxt
    again, _, _ = oracle.kmeans_step(k, lam, cb)
    np.testing.assert_allclose(again, cb, rtol=1e-13, atol=1e-15)


# --------------------------------------------------------------------------- codes wider than 8 bits, shared codebook
# (Sec. 2.2: one codebook of 2^b centroids, (d_h / d) x (b / 8) bytes of indices per vector; Sec. 4.1 / Tables 1-3:
#  d8b12, d4b12, K-d4b10 / V-d8b12; Sec. 4.4: codebook size 2^12 x 8 x 2 bytes for 1.5 bits)

def test_pack_codes_worked_example_and_big_integer_definition(oracle):
    """The row is one little-endian bit string: code m sits at bits m*b .. m*b + b - 1."""
    # by hand: 0xABC then 0x123 at 12 bits = the 24-bit number 0x123ABC = bytes BC 3A 12
    np.testing.assert_array_equal(oracle.pack_codes(np.array([[0xABC, 0x123]], dtype=np.uint16), 12),
                                  np.array([[0xBC, 0x3A, 0x12]], dtype=np.uint8))
    # 10 bits: 0x3FF, 0, 0x155, 0x2AA -> 0x2AA << 30 | 0x155 << 20 | 0 << 10 | 0x3FF
    v = (0x2AA << 30) | (0x155 << 20) | 0x3FF
    np.testing.assert_array_equal(oracle.pack_codes(np.array([0x3FF, 0, 0x155, 0x2AA], dtype=np.uint16), 10),
                                  np.frombuffer(v.to_bytes(5, "little"), dtype=np.uint8))
    g = synth.rng(77)
    for bits, M in ((12, 16), (10, 32), (12, 32), (10, 16), (8, 32)):
        idx = g.integers(0, 1 << bits, size=(3, 5, M), dtype=np.uint16)
        packed = oracle.pack_codes(idx, bits)
        assert packed.dtype == np.uint8 and packed.shape == (3, 5, M * bits // 8)
        for row, prow in zip(idx.reshape(-1, M), packed.reshape(-1, M * bits // 8)):
            big = sum(int(c) << (m * bits) for m, c in enumerate(row))         # Python big integer
            assert bytes(prow) == big.to_bytes(M * bits // 8, "little")
        np.testing.assert_array_equal(oracle.unpack_codes(packed, bits, M), idx)
    # 8-bit codes: the packed row is the code row itself
    idx8 = g.integers(0, 256, size=(4, 32), dtype=np.uint16)
    np.testing.assert_array_equal(oracle.pack_codes(idx8, 8), idx8.astype(np.uint8))


@pytest.mark.parametrize("d,C", [(8, 4096), (4, 1024), (4, 4096), (8, 1024)])
def test_shared_codebook_encode_vs_cdist_brute_force(oracle, d, C):
    """Eq. 2 with one codebook for every sub-space: each sub-vector against the same C centroids."""
    g = synth.rng(300 + d + C)
    D, N = 32, 40
    M = D // d
    X = g.standard_normal((N, D))
    cb = g.standard_normal((1, C, d))
    idx, gap = oracle.vq_encode(X, cb, want_gap=True)
    assert idx.dtype == np.uint16 and idx.shape == (N, M)
    dist = scipy.spatial.distance.cdist(X.reshape(N * M, d), cb[0], metric="sqeuclidean")
    np.testing.assert_array_equal(idx.reshape(-1), dist.argmin(axis=1))
    two = np.sort(dist, axis=1)[:, :2]
    np.testing.assert_allclose(gap.reshape(-1), (two[:, 1] - two[:, 0]) / two[:, 0], rtol=1e-9)
    # sub-vectors that are centroids come back as their own (lowest duplicate) index; ties -> lowest index
    cb[0, 700] = cb[0, 5]
    pick = g.integers(0, C, size=(N, M))
    Xc = cb[0][pick].reshape(N, D)
    back = oracle.vq_encode(Xc, cb)
    np.testing.assert_array_equal(back, np.where(pick == 700, 5, pick))
    # dequantization is the table lookup
    np.testing.assert_array_equal(oracle.vq_dequantize(back, cb), cb[0][back].reshape(N, D))


def test_general_encode_reduces_to_the_per_sub_space_one(oracle):
    """A shared codebook replicated M times is a per-sub-space codebook: both forms must agree,
    and the uint16 path with 256 centroids must reproduce the uint8 path."""
    g = synth.rng(311)
    D, d, C, N = 64, 4, 256, 33
    M = D // d
    X = g.standard_normal((N, D))
    shared = g.standard_normal((1, C, d))
    a = oracle.vq_encode(X, shared)                                     # general path (Mcb = 1)
    b = oracle.vq_encode(X, np.repeat(shared, M, axis=0))               # uint8 path
    assert a.dtype == np.uint16 and b.dtype == np.uint8
    np.testing.assert_array_equal(a, b)


def test_wide_encode_keys_vs_numpy_pipeline(oracle):
    """Keys: smooth, rotate (library Hadamard), then the shared-codebook search, batch layout."""
    g = synth.rng(312)
    B, Hkv, T, D, d, C = 2, 2, 9, 128, 8, 4096
    k = g.standard_normal((B, Hkv, T, D)).astype(np.float16)
    lam = np.exp(0.5 * g.standard_normal((Hkv, D))).astype(np.float32)
    cb = g.standard_normal((Hkv, 1, C, d)).astype(np.float16)
    got, gap = oracle.encode_keys(k, lam, cb, want_gap=True)
    gotv = oracle.encode_values(k, cb)
    assert got.dtype == np.uint16 and got.shape == (B, Hkv, T, D // d)
    H = scipy.linalg.hadamard(D) / np.sqrt(D)
    for b in range(B):
        for h in range(Hkv):
            Kt = (k[b, h].astype(np.float64) / lam[h].astype(np.float64)) @ H
            dist = scipy.spatial.distance.cdist(Kt.reshape(-1, d), cb[h, 0].astype(np.float64), "sqeuclidean")
            ok = (dist.argmin(axis=1) == got[b, h].reshape(-1)) | (gap[b, h].reshape(-1) < 1e-9)
            assert ok.all()
            dist = scipy.spatial.distance.cdist(k[b, h].astype(np.float64).reshape(-1, d),
                                                cb[h, 0].astype(np.float64), "sqeuclidean")
            np.testing.assert_array_equal(dist.argmin(axis=1), gotv[b, h].reshape(-1))


@pytest.mark.parametrize("kcfg,vcfg", [((8, 4096, 1), (8, 4096, 1)), ((4, 1024, 1), (8, 4096, 1)),
                                       ((8, 4096, 1), (8, 256, 16)), ((4, 256, 32), (4, 4096, 1))])
def test_wide_decode_matches_torch_sdpa_on_dequantized_cache(oracle, kcfg, vcfg):
    """Eq. 10 with wide codes / shared codebooks is textbook attention on the looked-up rows;
    keys and values mix code widths and sharing."""
    g = synth.rng(320 + kcfg[1] + vcfg[1])
    B, Hq, Hkv, D, N = 2, 4, 2, 128, 61
    G = Hq // Hkv
    (d_k, C_k, Mcb_k), (d_v, C_v, Mcb_v) = kcfg, vcfg
    Mk, Mv = D // d_k, D // d_v
    cb_k = g.standard_normal((Hkv, Mcb_k, C_k, d_k)).astype(np.float16)
    cb_v = g.standard_normal((Hkv, Mcb_v, C_v, d_v)).astype(np.float16)
    k_idx = g.integers(0, C_k, size=(B, Hkv, N, Mk), dtype=np.uint16)
    v_idx = g.integers(0, C_v, size=(B, Hkv, N, Mv), dtype=np.uint16)
    q = g.standard_normal((B, Hq, D)).astype(np.float16)
    lam = np.exp(0.5 * g.standard_normal((Hkv, D))).astype(np.float32)
    seq = np.array([61, 17])
    out, lse = oracle.decode_attention(q, lam, cb_k, cb_v, k_idx, v_idx, seq)
    Hm = scipy.linalg.hadamard(D) / np.sqrt(D)

    def rows(idx, cb):          # numpy fancy indexing, not the oracle's loop
        M = idx.shape[1]
        tab = cb.astype(np.float64)
        return (tab[0][idx] if tab.shape[0] == 1 else tab[np.arange(M)[None, :], idx]).reshape(idx.shape[0], -1)

    for b in range(B):
        n = seq[b]
        Kh = np.stack([rows(k_idx[b, h, :n], cb_k[h]) for h in range(Hkv)])
        Vh = np.stack([rows(v_idx[b, h, :n], cb_v[h]) for h in range(Hkv)])
        qt = (q[b].astype(np.float64) * np.repeat(lam.astype(np.float64), G, axis=0)) @ Hm
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(qt)[None, :, None, :],
            torch.from_numpy(Kh).repeat_interleave(G, dim=0)[None],
            torch.from_numpy(Vh).repeat_interleave(G, dim=0)[None])[0, :, 0].numpy()
        np.testing.assert_allclose(out[b], ref, rtol=1e-11, atol=1e-13)
        scores = np.einsum("hd,hnd->hn", qt, np.repeat(Kh, G, axis=0)) / np.sqrt(D)
        np.testing.assert_allclose(lse[b], scipy.special.logsumexp(scores, axis=1), rtol=1e-12)


def test_wide_residual_window_matches_sdpa_on_concatenated_cache(oracle):
    """Sec. 4.1's full-precision window with a wide-code cache: attention over the looked-up rows
    followed by the raw window rows, window keys carried into the transformed domain (Eq. 7)."""
    g = synth.rng(341)
    B, Hq, Hkv, D, N, R = 2, 4, 2, 128, 37, 9
    G = Hq // Hkv
    cb_k = g.standard_normal((Hkv, 1, 4096, 8)).astype(np.float16)
    cb_v = g.standard_normal((Hkv, 16, 256, 8)).astype(np.float16)
    k_idx = g.integers(0, 4096, size=(B, Hkv, N, 16), dtype=np.uint16)
    v_idx = g.integers(0, 256, size=(B, Hkv, N, 16), dtype=np.uint16)
    q = g.standard_normal((B, Hq, D)).astype(np.float16)
    lam = np.exp(0.5 * g.standard_normal((Hkv, D))).astype(np.float32)
    k_res = g.standard_normal((B, Hkv, R, D)).astype(np.float16)
    v_res = g.standard_normal((B, Hkv, R, D)).astype(np.float16)
    seq, res = np.array([37, 12]), np.array([9, 4])
    out, lse = oracle.decode_attention_residual(q, lam, cb_k, cb_v, k_idx, v_idx, k_res, v_res, seq, res)
    Hm = scipy.linalg.hadamard(D) / np.sqrt(D)
    for b in range(B):
        n, r = seq[b], res[b]
        Kh = np.stack([cb_k[h, 0].astype(np.float64)[k_idx[b, h, :n]].reshape(n, D) for h in range(Hkv)])
        Vh = np.stack([cb_v[h].astype(np.float64)[np.arange(16)[None, :], v_idx[b, h, :n]].reshape(n, D)
                       for h in range(Hkv)])
        Kw = np.stack([(k_res[b, h, :r].astype(np.float64) / lam[h].astype(np.float64)) @ Hm for h in range(Hkv)])
        Kall = np.concatenate([Kh, Kw], axis=1)
        Vall = np.concatenate([Vh, v_res[b, :, :r].astype(np.float64)], axis=1)
        qt = (q[b].astype(np.float64) * np.repeat(lam.astype(np.float64), G, axis=0)) @ Hm
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(qt)[None, :, None, :],
            torch.from_numpy(Kall).repeat_interleave(G, dim=0)[None],
            torch.from_numpy(Vall).repeat_interleave(G, dim=0)[None])[0, :, 0].numpy()
        np.testing.assert_allclose(out[b], ref, rtol=1e-10, atol=1e-12)
        scores = np.einsum("hd,hnd->hn", qt, np.repeat(Kall, G, axis=0)) / np.sqrt(D)
        np.testing.assert_allclose(lse[b], scipy.special.logsumexp(scores, axis=1), rtol=1e-11)


def test_shared_codebook_kmeans_update_matches_scipy_on_pooled_sub_vectors(oracle):
    """One Lloyd iteration for a codebook shared by the sub-spaces = scipy's kmeans2 (one iteration,
    given initial centroids) on the sub-vectors of all sub-spaces pooled; empty clusters keep theirs."""
    import scipy.cluster.vq
    g = synth.rng(351)
    N, D, d, C = 90, 32, 8, 1024
    M = D // d
    X = g.standard_normal((N, D))
    cb = g.standard_normal((1, C, d))
    idx = oracle.vq_encode(X, cb)
    new, counts = oracle.kmeans_update(X, idx, cb)
    assert new.shape == (1, C, d) and counts.shape == (1, C) and counts.sum() == N * M
    import warnings
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")                 # scipy warns about the empty clusters
        ref, labels = scipy.cluster.vq.kmeans2(X.reshape(N * M, d), cb[0].copy(), iter=1, minit="matrix",
                                               missing="warn")
    np.testing.assert_array_equal(labels, idx.reshape(-1))
    np.testing.assert_array_equal(counts[0], np.bincount(labels, minlength=C))
    used = counts[0] > 0
    assert used.sum() < C                               # the case has empty clusters
    np.testing.assert_allclose(new[0][used], ref[used], rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(new[0][~used], cb[0][~used])
    # batch driver: per KV head, keys transformed first; monotone error over iterations
    B, Hkv, T, Dk = 1, 2, 300, 128
    k, _ = synth.keys_with_outlier_channels(g, B, Hkv, T, Dk, 2)
    lam = np.stack([oracle.smoothing_factors(k[:, h]) for h in range(Hkv)])
    cbk = g.standard_normal((Hkv, 1, 1024, 8))

    def error(cbx):
        idx = oracle.encode_keys(k, lam, cbx)
        return sum(((oracle.transform_keys(k[0, h].astype(np.float64), lam[h])
                     - oracle.vq_dequantize(idx[0, h], cbx[h])) ** 2).sum() for h in range(Hkv))

    errs = [error(cbk)]
    for _ in range(3):
        cbk, cnt, _ = oracle.kmeans_step(k, lam, cbk)
        assert cnt.shape == (Hkv, 1, 1024) and cnt.sum() == Hkv * T * 16
        errs.append(error(cbk))
    assert all(b <= a * (1 + 1e-12) for a, b in zip(errs, errs[1:])) and errs[-1] < 0.9 * errs[0]


def test_wide_decode_special_cases(oracle):
    """q = 0: the mean of the looked-up value rows and L = ln N; N = 1: that token's value row."""
    g = synth.rng(333)
    B, Hq, Hkv, D, N, d, C = 1, 2, 1, 128, 23, 8, 4096
    cb_k = g.standard_normal((Hkv, 1, C, d)).astype(np.float16)
    cb_v = g.standard_normal((Hkv, 1, C, d)).astype(np.float16)
    k_idx = g.integers(0, C, size=(B, Hkv, N, D // d), dtype=np.uint16)
    v_idx = g.integers(0, C, size=(B, Hkv, N, D // d), dtype=np.uint16)
    lam = np.ones((Hkv, D), dtype=np.float32)
    Vh = cb_v[0, 0].astype(np.float64)[v_idx[0, 0]].reshape(N, D)
    out, lse = oracle.decode_attention(np.zeros((B, Hq, D), np.float16), lam, cb_k, cb_v, k_idx, v_idx)
    np.testing.assert_allclose(out[0, 0], Vh.mean(axis=0), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, np.log(N), rtol=1e-13)
    q = g.standard_normal((B, Hq, D)).astype(np.float16)
    out1, lse1 = oracle.decode_attention(q, lam, cb_k, cb_v, k_idx, v_idx, np.array([1]))
    np.testing.assert_allclose(out1[0, 1], Vh[0], rtol=1e-13)
    Kh0 = cb_k[0, 0].astype(np.float64)[k_idx[0, 0, 0]].reshape(D)
    H = scipy.linalg.hadamard(D) / np.sqrt(D)
    np.testing.assert_allclose(lse1[0, 1], ((q[0, 1].astype(np.float64)) @ H) @ Kh0 / np.sqrt(D), rtol=1e-11)


def test_decode_rejects_empty_sequence(oracle):
    s, x = _small_decode_case(28, B=2)
    with pytest.raises(ValueError):
        oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"], np.array([5, 0]))


def test_tiny_config_end_to_end_quantization_is_sane(oracle):
    """Config 1 (1 head, N 4096, outlier keys): the quantized attention stays close to the
    full-precision attention of Eq. 1 -- a coarse end-to-end check that encode and decode agree
    on the side of the transform (a swapped lambda or a missing Hadamard breaks it)."""
    sh = synth.TINY
    e = synth.encode_inputs(sh, seed=1, n_outlier=4)
    K = e["k"][0, 0].astype(np.float64)
    V = e["v"][0, 0].astype(np.float64)
    lam = oracle.smoothing_factors(K)[None, :]
    # codebooks fitted to the data's own scale so that quantization error is small
    Kt = oracle.transform_keys(K, lam[0])
    g = synth.rng(99)
    cb_k = np.stack([Kt[g.choice(sh.N, 256, replace=False), 4 * m:4 * m + 4] for m in range(32)])[None]
    cb_v = np.stack([V[g.choice(sh.N, 256, replace=False), 4 * m:4 * m + 4] for m in range(32)])[None]
    k_idx = oracle.encode_keys(e["k"], lam, cb_k)
    v_idx = oracle.encode_values(e["v"], cb_v)
    out, _ = oracle.decode_attention(e["q"], lam, cb_k, cb_v, k_idx, v_idx)
    q = e["q"][0, 0].astype(np.float64)
    p = scipy.special.softmax(K @ q / np.sqrt(sh.D))
    full = p @ V
    # scores of the quantized cache correlate strongly with the exact ones
    s_q = oracle.vq_dequantize(k_idx[0, 0], cb_k[0]) @ oracle.transform_query(q, lam[0]) / np.sqrt(sh.D)
    assert np.corrcoef(s_q, K @ q / np.sqrt(sh.D))[0, 1] > 0.9
    assert np.abs(out[0, 0] - full).max() < 0.5 * np.abs(V).max()


# --------------------------------------------------------------------------- K-Means training loop (Sec. 2.2, 4.1)

def test_kmeans_train_matches_scipy_kmeans2_over_k_iterations(oracle):
    """The training loop with no early stop and no fp16 rounding is scipy's kmeans2 started from the
    same centroids and run for the same number of iterations (values: no transform; one KV head,
    one sub-space per column block), labels and centroids; the error it reports for an iteration is
    the distortion of that iteration's assignment."""
    import warnings
    from scipy.cluster.vq import kmeans2
    g = synth.rng(91)
    for d, iters in ((4, 5), (2, 3), (8, 4)):
        D, T = 2 * d, 1500
        v = (g.standard_normal((1, 1, T, D)) * np.array([1.0, 0.3] * d)).astype(np.float16)
        init = (g.standard_normal((1, D // d, 256, d)) * 0.8).astype(np.float16).astype(np.float64)
        init[0, 0, 9] = 40.0                                  # stays empty in every iteration
        cb, counts, idx, errs = oracle.kmeans_train(v, None, init, max_iters=iters, tol=-1.0, round_f16=False)
        assert len(errs) == iters and counts[0, 0, 9] == 0 and (cb[0, 0, 9] == 40.0).all()
        X = v[0, 0].astype(np.float64)
        for m in range(D // d):
            with warnings.catch_warnings():
                warnings.simplefilter("ignore")
                ref, _ = kmeans2(X[:, m * d:(m + 1) * d], init[0, m].copy(), iter=iters, minit="matrix")
                # the labels scipy returns belong to the centroids BEFORE its last update: the loop's idx
                before, lab = kmeans2(X[:, m * d:(m + 1) * d], init[0, m].copy(), iter=iters - 1, minit="matrix") \
                    if iters > 1 else (init[0, m], None)
            np.testing.assert_allclose(cb[0, m], ref, rtol=1e-10, atol=1e-12)
            dist = ((X[:, None, m * d:(m + 1) * d] - before[None]) ** 2).sum(-1)
            np.testing.assert_array_equal(idx[0, 0, :, m], dist.argmin(1))
        # errors: distortion of each iteration's assignment, by brute force on the first and the last
        cb1, _, idx1, e1 = oracle.kmeans_train(v, None, init, max_iters=1, tol=-1.0, round_f16=False)
        want = sum(((X[:, None, m * d:(m + 1) * d] - init[0, m][None]) ** 2).sum(-1).min(1).sum() for m in range(D // d))
        np.testing.assert_allclose(e1[0], want, rtol=1e-12)
        np.testing.assert_allclose(errs[0], want, rtol=1e-12)
        assert all(b <= a * (1 + 1e-12) for a, b in zip(errs, errs[1:]))


def test_kmeans_train_stopping_rule_and_fp16_storage(oracle):
    """Well separated clusters: the error stops improving after a few iterations and the loop ends
    there (far before 30); tol < 0 runs all iterations; with fp16 storage every returned centroid is
    an fp16 number and the trajectory equals stepping by hand with the rounding in between."""
    g = synth.rng(92)
    B, Hkv, T, D, d = 1, 2, 1200, 16, 4
    centers = g.standard_normal((Hkv, D // d, 8, d)) * 4.0
    pick = g.integers(0, 8, size=(B, Hkv, T, D // d))
    k = np.empty((B, Hkv, T, D))
    for h in range(Hkv):
        for m in range(D // d):
            k[:, h, :, m * d:(m + 1) * d] = centers[h, m][pick[:, h, :, m]] + 0.05 * g.standard_normal((B, T, d))
    k = k.astype(np.float16)
    cb0 = synth.codebooks(g, Hkv, D // d, d)
    cb, counts, idx, errs = oracle.kmeans_train(k, None, cb0, max_iters=30, tol=1e-4)
    assert 2 <= len(errs) < 30
    assert errs[-2] - errs[-1] <= 1e-4 * errs[-2] and all(a - b > 1e-4 * a for a, b in zip(errs[:-2], errs[1:-1]))
    np.testing.assert_array_equal(cb, cb.astype(np.float16).astype(np.float64))
    # by hand
    c = cb0.astype(np.float64)
    for t in range(len(errs)):
        new, cnt, ix = oracle.kmeans_step(k, None, c)
        np.testing.assert_allclose(oracle.quantization_error(k, None, c, ix).sum(), errs[t], rtol=1e-13)
        c = new.astype(np.float16).astype(np.float64)
    np.testing.assert_array_equal(c, cb)
    np.testing.assert_array_equal(ix, idx)
    np.testing.assert_array_equal(cnt, counts)
    full = oracle.kmeans_train(k, None, cb0, max_iters=7, tol=-1.0)
    assert len(full[3]) == 7
    # keys: trained on the transformed keys (Sec. 3.2); the error is measured there too
    lam = np.stack([oracle.smoothing_factors(k[:, h]) for h in range(Hkv)])
    cbk, _, ixk, ek = oracle.kmeans_train(k, lam, cb0, max_iters=3, tol=-1.0)
    rows = oracle.transform_keys(k[0, 0].astype(np.float64), lam[0])
    first = oracle.encode_keys(k, lam, cb0.astype(np.float64))
    e0 = oracle.quantization_error(k, lam, cb0.astype(np.float64), first)
    np.testing.assert_allclose(e0.sum(), ek[0], rtol=1e-13)
    np.testing.assert_allclose(e0[0], ((rows - oracle.vq_dequantize(first[0, 0], cb0[0].astype(np.float64))) ** 2).sum(),
                               rtol=1e-13)
