"""vecinfer_decode_attention_static (the entry point that allocates nothing: split partials in a
fixed array inside the library) against vecinfer_decode_attention on the same inputs, through the
C ABI.  Same kernels, so the results must be bit-identical; the oracle bar is checked as well.
Two calls in a row share the one array, the second on a smaller input (stale partials of the
first call stay behind it and must not be read)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_06175_amd import binding as vb
from paper_2510_06175_amd import synth

from helpers import LSE_ATOL, OUT_RTOL_INF, cfg_of, dev, oracle_view

pytestmark = pytest.mark.gpu


def _both(shape, seed, splits, seq_lens=None):
    x = synth.decode_inputs(shape, seed=seed)
    cfg = cfg_of(shape)
    t = {k: dev(v) for k, v in x.items()}
    sl = None if seq_lens is None else torch.as_tensor(seq_lens, dtype=torch.int32).cuda()
    res = []
    for static in (False, True):
        out = torch.full((shape.B, shape.Hq, shape.D), float("nan"), dtype=torch.float16, device="cuda")
        lse = torch.full((shape.B, shape.Hq), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            vb.vecinfer_decode_attention_static(cfg, t["q"], t["lam"], t["cb_k"], t["cb_v"], t["k_idx"], t["v_idx"],
                                                out, lse=lse, seq_lens=sl, num_splits=splits)
        else:
            ws = vb.new_workspace(cfg, shape.B, shape.N, splits)
            vb.vecinfer_decode_attention(cfg, t["q"], t["lam"], t["cb_k"], t["cb_v"], t["k_idx"], t["v_idx"], ws,
                                         out, lse=lse, seq_lens=sl, num_splits=splits)
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), lse.cpu().numpy()))
    (o_ws, l_ws), (o_st, l_st) = res
    np.testing.assert_array_equal(o_st, o_ws)
    np.testing.assert_array_equal(l_st, l_ws)
    ox = oracle_view(shape, x)
    ref_o, ref_l = oracle.decode_attention(ox["q"], ox["lam"], ox["cb_k"], ox["cb_v"], ox["k_idx"], ox["v_idx"],
                                           seq_lens=seq_lens)
    err = np.abs(o_st.astype(np.float64) - ref_o).max(axis=-1)
    assert (err <= OUT_RTOL_INF * np.abs(ref_o).max(axis=-1)).all()
    assert np.abs(l_st - ref_l).max() <= LSE_ATOL


def test_static_scratch_two_calls_second_smaller():
    # first call: 64 splits of a GQA batch (1.1 MB of partials); second: fewer tokens, fewer heads,
    # fewer splits, so most of the first call's partials stay in the array behind it
    _both(synth.Shape(2, 32, 8, 128, 9000, 4, 4), seed=11, splits=64, seq_lens=[9000, 4100])
    _both(synth.Shape(1, 8, 2, 128, 1300, 4, 4), seed=12, splits=5)
    # and a third with automatic splits and 12-bit codes
    _both(synth.Shape(1, 8, 2, 128, 3000, 8, 8, 12, 12), seed=13, splits=0)


def test_static_scratch_refuses_what_does_not_fit():
    shape = synth.Shape(8, 32, 8, 128, 4096, 4, 4)
    cfg = cfg_of(shape)
    assert vb.vecinfer_decode_workspace_bytes(cfg, shape.B, shape.N, 64) > vb.STATIC_SCRATCH_BYTES
    x = synth.decode_inputs(shape, seed=3)
    t = {k: dev(v) for k, v in x.items()}
    out = torch.zeros((shape.B, shape.Hq, shape.D), dtype=torch.float16, device="cuda")
    with pytest.raises(vb.VecInferError) as e:
        vb.vecinfer_decode_attention_static(cfg, t["q"], t["lam"], t["cb_k"], t["cb_v"], t["k_idx"], t["v_idx"], out,
                                            num_splits=64)
    assert e.value.code == vb.EWORKSPACE
    torch.cuda.synchronize()
    assert (out == 0).all()
