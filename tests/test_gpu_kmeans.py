"""GPU parity of vecinfer_kmeans_train (Sec. 2.2: K-Means builds the codebooks; Sec. 3.2: on the
transformed keys and the original values; Sec. 4.1: at most 30 iterations) against the oracle's
kmeans_train / kmeans_step / quantization_error, through the C ABI.

The cluster sums are fp32 atomics, so two runs may round a centroid to neighbouring fp16 values and
then part slowly.  What is exact is therefore checked iteration by iteration from the state the GPU
itself was in (calls of one iteration each, in place); calls of several iterations are checked by
what does not depend on the path (the means of the last assignment, the counts, the sizes) and by
the errors, which are smooth in the codebook.
"""
import numpy as np
import pytest
import torch

from paper_2510_06175_amd import synth
import oracle
from paper_2510_06175_amd import binding as vb
from helpers import cfg_of, dev, assert_indices_match

pytestmark = pytest.mark.gpu


def _problem(shape, kind, seed):
    e = synth.encode_inputs(shape, seed=seed, n_outlier=3)
    if kind == "keys":
        lam = np.stack([oracle.smoothing_factors(e["k"][:, h]) for h in range(shape.Hkv)]).astype(np.float32)
        return e["k"], lam, e["cb_k"]
    return e["v"], None, e["cb_v"]


class Trainer:
    """Device buffers of one training problem; train() runs the entry point in place."""

    def __init__(self, shape, x, lam, cb0):
        self.cfg = cfg_of(shape)
        self.keys = lam is not None
        B, Hkv, T, D = x.shape
        self.bits = shape.b_k if self.keys else shape.b_v
        self.M = shape.Mk if self.keys else shape.Mv
        self.x, self.lam = dev(x), None if lam is None else dev(lam)
        self.cb = dev(cb0).clone()
        self.codes = torch.full((B, Hkv, T, self.cfg.row_bytes(self.keys)), 0xEE, dtype=torch.uint8, device="cuda")
        self.counts = torch.full(tuple(cb0.shape[:-1]), -1, dtype=torch.int32, device="cuda")
        self.ws = vb.new_kmeans_workspace(self.cfg, self.keys)
        self.ws.fill_(0xA5)                      # the library clears what must start at zero

    def train(self, max_iters, tol):
        iters = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        errors = torch.full((max_iters,), float("nan"), dtype=torch.float64, device="cuda")
        vb.vecinfer_kmeans_train(self.cfg, self.x, self.lam, self.cb, self.codes, self.ws, counts=self.counts,
                                 max_iters=max_iters, tol=tol, iters_run=iters, errors=errors)
        torch.cuda.synchronize()
        return int(iters.item()), errors.cpu().numpy()

    def state(self):
        """(codebook, codes unpacked to [B, Hkv, T, M], counts); a shared table as [Hkv, 1, C, d] / [Hkv, 1, C],
        the oracle's form."""
        cb, counts = self.cb.cpu().numpy(), self.counts.cpu().numpy()
        if self.bits != 8:
            cb, counts = cb[:, None], counts[:, None]
        return cb, oracle.unpack_codes(self.codes.cpu().numpy(), self.bits, self.M), counts


def _rows(x, lam, g):
    B, Hkv, T, D = x.shape
    rows = x[:, g].reshape(B * T, D).astype(np.float64)
    return rows if lam is None else oracle.transform_keys(rows, lam[g])


def _check_means(x, lam, cb_after, codes, counts, what, cb_before=None):
    """cb_after = the means of the clusters codes defines (fp32 sums, fp16 result: one fp16 ulp);
    counts exact; with cb_before, empty clusters kept bit for bit."""
    B, Hkv, T, D = x.shape
    for g in range(Hkv):
        base = cb_after[g] if cb_before is None else cb_before[g]
        ref_cb, ref_counts = oracle.kmeans_update(_rows(x, lam, g), codes[:, g].reshape(B * T, -1), base)
        np.testing.assert_array_equal(counts[g], ref_counts)
        full = ref_counts > 0
        np.testing.assert_allclose(cb_after[g][full].astype(np.float64), ref_cb[full], rtol=1.5e-3, atol=1e-6,
                                   err_msg=f"{what}: centroids of head {g}")
        if cb_before is not None:
            np.testing.assert_array_equal(cb_after[g][~full], cb_before[g][~full])


SHAPES = [synth.Shape(2, 4, 2, 128, 1000, 4, 4), synth.Shape(1, 2, 2, 64, 777, 2, 8),
          synth.Shape(3, 1, 1, 128, 70, 8, 2),
          # 10- / 12-bit codes: one shared codebook per KV head, trained on the pooled sub-vectors
          synth.Shape(2, 2, 2, 128, 300, 8, 4, 12, 10), synth.Shape(1, 2, 2, 64, 330, 4, 8, 10, 12),
          synth.Shape(1, 2, 2, 128, 260, 8, 8, 10, 10)]


@pytest.mark.parametrize("kind", ["keys", "values"])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: f"B{s.B}g{s.Hkv}D{s.D}T{s.N}k{s.d_k}b{s.b_k}v{s.d_v}b{s.b_v}")
def test_train_iteration_by_iteration(shape, kind):
    """Five calls of one iteration each, in place.  Every call: the assignment is the oracle's for
    the codebook the call started from (Eq. 2, near-ties logged), the error is the oracle's for that
    codebook and the GPU's assignment, the new centroids are the means within one fp16 ulp."""
    x, lam, cb0 = _problem(shape, kind, seed=shape.N + 11)
    cb0 = cb0.copy()
    cb0[..., 9, :] = 300.0                                 # a centroid nobody is assigned to
    t = Trainer(shape, x, lam, cb0)
    before = cb0 if t.bits == 8 else cb0[:, None]
    errs = []
    for it in range(5):
        n, e = t.train(1, 1e-4)
        assert n == 1
        after, codes, counts = t.state()
        if lam is not None:
            ref_idx, gap = oracle.encode_keys(x, lam, before, want_gap=True)
        else:
            ref_idx, gap = oracle.encode_values(x, before, want_gap=True)
        assert_indices_match(codes, ref_idx, gap, f"train {kind} iteration {it}: assignment")
        ref_e = oracle.quantization_error(x, lam, before, codes).sum()
        assert abs(e[0] - ref_e) <= 2e-5 * ref_e, (it, e[0], ref_e)
        _check_means(x, lam, after, codes, counts, f"train {kind} iteration {it}", cb_before=before)
        errs.append(e[0])
        before = after
    assert all(b <= a * (1 + 1e-3) for a, b in zip(errs, errs[1:])), errs
    assert errs[-1] < errs[0]


def _clear_tol(errors, lo=3):
    """A tolerance between two consecutive relative improvements of an error sequence that differ
    by a clear factor, so that rounding cannot move the iteration the rule stops at; returns
    (tol, iterations the rule then runs)."""
    r = (errors[:-1] - errors[1:]) / errors[:-1]           # r[t-1] = improvement of iteration t
    for t in range(lo, len(r)):
        if r[t] < r[t - 1] / 1.3 and all(r[:t] > 1.15 * np.sqrt(r[t] * r[t - 1])):
            return float(np.sqrt(r[t] * r[t - 1])), t + 2  # stops after iteration t + 1
    raise AssertionError("no clear gap in the improvements")


@pytest.mark.parametrize("kind", ["keys", "values"])
def test_train_stopping_rule_and_errors(kind):
    """One call of up to 30 iterations against the oracle's loop: the same number of iterations for
    a tolerance that sits clearly between two improvements, the errors within 1e-3 (fp16 codebooks
    that may differ by an ulp here and there), later error slots untouched, and the final state
    self-consistent (means of the last assignment, counts)."""
    shape = synth.Shape(2, 4, 2, 128, 1500, 4, 4)
    x, lam, cb0 = _problem(shape, kind, seed=91)
    _, _, _, free = oracle.kmeans_train(x, lam, cb0, max_iters=12, tol=-1.0)
    tol, n_ref = _clear_tol(free)
    ref_cb, ref_counts, ref_idx, ref_err = oracle.kmeans_train(x, lam, cb0, max_iters=30, tol=tol)
    assert len(ref_err) == n_ref < 12
    t = Trainer(shape, x, lam, cb0)
    n, e = t.train(30, tol)
    assert n == n_ref, (n, n_ref, e[:n], ref_err)
    np.testing.assert_allclose(e[:n], ref_err, rtol=1e-3)
    assert np.isnan(e[n:]).all()
    cb, codes, counts = t.state()
    _check_means(x, lam, cb, codes, counts, f"train {kind}")
    assert counts.sum() == codes.size
    # the centroids of the oracle's run: the same up to the ulp-level partings described above
    close = np.isclose(cb.astype(np.float64), ref_cb, rtol=2e-3, atol=1e-6)
    assert close.mean() > 0.98, close.mean()
    assert (codes == ref_idx).mean() > 0.98
    # the codebook the GPU ended with is as good as the oracle's (error of a fresh assignment)
    enc = (lambda c: oracle.encode_keys(x, lam, c)) if lam is not None else (lambda c: oracle.encode_values(x, c))
    e_gpu = oracle.quantization_error(x, lam, cb, enc(cb)).sum()
    e_ref = oracle.quantization_error(x, lam, ref_cb, enc(ref_cb)).sum()
    assert abs(e_gpu - e_ref) <= 1e-3 * e_ref


def test_train_runs_all_iterations_without_a_tolerance():
    """tol < 0 never stops early; a huge tol stops after the second iteration (the first one that
    has a predecessor); max_iters = 1 never looks at the rule; a call equals the chain of
    single-iteration calls up to the atomics' rounding."""
    shape = synth.Shape(1, 2, 2, 128, 640, 4, 4)
    x, lam, cb0 = _problem(shape, "values", seed=5)
    t = Trainer(shape, x, lam, cb0)
    n, e = t.train(7, -1.0)
    assert n == 7 and np.isfinite(e).all()
    cb7 = t.state()[0]
    chain = Trainer(shape, x, lam, cb0)
    e_chain = [chain.train(1, -1.0)[1][0] for _ in range(7)]
    np.testing.assert_allclose(e, e_chain, rtol=1e-3)
    assert np.isclose(cb7.astype(np.float64), chain.state()[0].astype(np.float64), rtol=2e-3, atol=1e-6).mean() > 0.98
    t2 = Trainer(shape, x, lam, cb0)
    n, e2 = t2.train(30, 10.0)
    assert n == 2 and np.isnan(e2[2:]).all()
    np.testing.assert_allclose(e2[:2], e[:2], rtol=1e-3)
    cb, codes, counts = t2.state()
    _check_means(x, lam, cb, codes, counts, "stopped after two")
    # the work enqueued after the stop left the state of iteration 1: same as a call of two iterations
    t3 = Trainer(shape, x, lam, cb0)
    assert t3.train(2, -1.0)[0] == 2
    assert np.isclose(cb.astype(np.float64), t3.state()[0].astype(np.float64), rtol=2e-3, atol=1e-6).mean() > 0.995


def test_train_one_iteration_equals_kmeans_step():
    shape = synth.Shape(2, 4, 2, 128, 1000, 4, 8)
    x, lam, cb0 = _problem(shape, "keys", seed=17)
    t = Trainer(shape, x, lam, cb0)
    t.train(1, 1e-4)
    cb, codes, counts = t.state()
    cb_out = torch.empty_like(t.cb)
    codes2 = torch.empty_like(t.codes)
    counts2 = torch.empty_like(t.counts)
    vb.vecinfer_kmeans_step(t.cfg, t.x, t.lam, dev(cb0), cb_out, codes2, t.ws, counts=counts2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(codes, codes2.cpu().numpy())
    np.testing.assert_array_equal(counts, counts2.cpu().numpy())
    got = cb_out.cpu().numpy()
    assert (got == cb).mean() > 0.999                       # the same sums up to the order of the atomics
    np.testing.assert_allclose(got.astype(np.float64), cb.astype(np.float64), rtol=1e-3, atol=1e-6)


def test_train_wide_codes_against_the_oracle_loop():
    """12-bit codes on sub-vectors of 8 (the 1.5-bit configuration): six iterations in one call against the
    oracle's loop on the shared codebook: errors, final means, counts."""
    shape = synth.Shape(2, 2, 2, 128, 400, 8, 8, 12, 12)
    x, lam, cb0 = _problem(shape, "keys", seed=23)
    ref_cb, ref_counts, ref_idx, ref_err = oracle.kmeans_train(x, lam, cb0[:, None], max_iters=6, tol=-1.0)
    t = Trainer(shape, x, lam, cb0)
    n, e = t.train(6, -1.0)
    assert n == 6
    np.testing.assert_allclose(e, ref_err, rtol=1e-3)
    cb, codes, counts = t.state()
    _check_means(x, lam, cb, codes, counts, "train d8b12")
    assert counts.sum() == codes.size
    assert (codes == ref_idx).mean() > 0.97


def test_train_full_size_iteration_properties():
    """65536 tokens x 8 KV heads, d = 4 (the size the iteration is timed at): three iterations in
    one call; the errors fall, the counts add up, and for sampled (KV head, sub-space) pairs the counts
    are the histogram of the codes and the centroids the means of their clusters."""
    shape = synth.Shape(1, 32, 8, 128, 65536, 4, 4)
    x, lam, cb0 = _problem(shape, "values", seed=3)
    t = Trainer(shape, x, lam, cb0)
    n, e = t.train(3, -1.0)
    assert n == 3 and e[0] >= e[1] * (1 - 1e-3) >= e[2] * (1 - 2e-3) > 0
    cb, codes, counts = t.state()
    assert (counts.sum(axis=2) == shape.N).all()
    rng = np.random.default_rng(0)
    for g, m in zip(rng.integers(0, shape.Hkv, 6), rng.integers(0, shape.Mv, 6)):
        sub = x[0, g, :, 4 * m:4 * m + 4].astype(np.float64)
        c = codes[0, g, :, m]
        np.testing.assert_array_equal(np.bincount(c, minlength=256), counts[g, m])
        sums = np.zeros((256, 4))
        np.add.at(sums, c, sub)
        full = counts[g, m] > 0
        np.testing.assert_allclose(cb[g, m][full].astype(np.float64), sums[full] / counts[g, m][full, None],
                                   rtol=1.5e-3, atol=1e-6)


@pytest.mark.parametrize("n_distinct", [1, 3, 40])
def test_train_heavily_shared_codes(n_distinct):
    """Tokens drawn from a handful of vectors: in every wavefront many lanes carry the same code, the
    case the accumulation resolves with one plain update and atomics for the rest.  Counts exact,
    means within one fp16 ulp, error against the oracle."""
    shape = synth.Shape(2, 2, 2, 128, 700, 4, 4)
    g = synth.rng(300 + n_distinct)
    pool = g.standard_normal((n_distinct, shape.D)).astype(np.float16)
    x = pool[g.integers(0, n_distinct, size=(shape.B, shape.Hkv, shape.N))]
    cb0 = g.standard_normal((shape.Hkv, shape.Mv, 256, shape.d_v)).astype(np.float16)
    t = Trainer(shape, x, None, cb0)
    n, e = t.train(1, -1.0)
    cb, codes, counts = t.state()
    ref_idx, gap = oracle.encode_values(x, cb0, want_gap=True)
    assert_indices_match(codes, ref_idx, gap, "shared codes: assignment")
    ref_e = oracle.quantization_error(x, None, cb0, codes).sum()
    assert abs(e[0] - ref_e) <= 2e-5 * ref_e
    _check_means(x, None, cb, codes, counts, "shared codes", cb_before=cb0)
    assert (counts > 0).sum(axis=2).max() <= n_distinct
