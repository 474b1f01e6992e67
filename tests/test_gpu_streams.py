"""The calls only enqueue work on the caller's stream: they run on a side stream, and a whole decode
step can be captured into a HIP graph (no allocation, no synchronisation, no host-side state that
changes between calls) and replayed with new inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_06175_amd import binding as vb
from paper_2510_06175_amd import synth

from helpers import assert_decode_close, cfg_of, dev

pytestmark = pytest.mark.gpu


def _alloc(shape):
    out = torch.full((shape.B, shape.Hq, shape.D), float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full((shape.B, shape.Hq), float("nan"), dtype=torch.float32, device="cuda")
    return out, lse


def test_calls_run_on_a_side_stream():
    shape = synth.Shape(2, 8, 2, 128, 3000, 4, 4)
    cfg = cfg_of(shape)
    x = synth.decode_inputs(shape, seed=11)
    ref = oracle.decode_attention(x["q"], x["lam"], x["cb_k"], x["cb_v"], x["k_idx"], x["v_idx"])
    host = {k: torch.from_numpy(np.ascontiguousarray(v)).pin_memory() for k, v in x.items()}
    side = torch.cuda.Stream()
    ws = vb.new_workspace(cfg, shape.B, shape.N)
    out, lse = _alloc(shape)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        # the inputs arrive on the side stream (asynchronous copies) right in front of the call:
        # only stream order makes them visible to the kernels
        t = {k: v.to("cuda", non_blocking=True) for k, v in host.items()}
        vb.vecinfer_decode_attention(cfg, t["q"], t["lam"], t["cb_k"], t["cb_v"], t["k_idx"], t["v_idx"], ws, out,
                                     lse=lse)
        explicit = _alloc(shape)
    # the same call with the stream passed explicitly instead of taken from torch's current one
    vb.vecinfer_decode_attention(cfg, t["q"], t["lam"], t["cb_k"], t["cb_v"], t["k_idx"], t["v_idx"], ws,
                                 explicit[0], lse=explicit[1], stream=side)
    side.synchronize()
    for o, l in ((out, lse), explicit):
        assert_decode_close(o.cpu().numpy().astype(np.float64), l.cpu().numpy().astype(np.float64), *ref,
                            what="side stream")


@pytest.mark.parametrize("shape", [synth.Shape(1, 8, 2, 128, 5000, 4, 4), synth.Shape(2, 8, 2, 128, 2500, 8, 8, 12, 12)],
                         ids=lambda s: f"k{s.d_k}b{s.b_k}")
def test_decode_step_in_a_hip_graph(shape):
    """Capture one whole step (append + attention + merge) and replay it with fresh queries and new
    tokens, with eager work and synchronisations in between; every replay must equal the eager call."""
    cfg = cfg_of(shape)
    x = synth.decode_inputs(shape, seed=21, n_cap=shape.N + 8)
    t = {k: dev(v) for k, v in x.items()}
    g = synth.rng(22)
    ws = vb.new_workspace(cfg, shape.B, shape.N + 8)
    q = t["q"].clone()
    k_new = torch.zeros((shape.B, shape.Hkv, 1, shape.D), dtype=torch.float16, device="cuda")
    v_new = torch.zeros_like(k_new)
    lens = torch.full((shape.B,), shape.N, dtype=torch.int32, device="cuda")
    out, lse = _alloc(shape)

    def step(o, l, k_idx, v_idx, sl):
        vb.vecinfer_decode_step(cfg, q, k_new, v_new, t["lam"], t["cb_k"], t["cb_v"], k_idx, v_idx, ws, o, lse=l,
                                seq_lens=sl, N=shape.N + 8)

    k_g, v_g = t["k_idx"].clone(), t["v_idx"].clone()
    step(out, lse, k_g, v_g, lens)                     # warm-up outside the capture (one-time kernel set-up)
    torch.cuda.synchronize()
    k_g.copy_(t["k_idx"]); v_g.copy_(t["v_idx"])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(out, lse, k_g, v_g, lens)
    k_e, v_e = t["k_idx"].clone(), t["v_idx"].clone()
    for it in range(4):
        # new inputs for this decode step: the sequences grow by one token
        q.copy_(dev(synth.queries(g, shape.B, shape.Hq, shape.D)))
        k_new.copy_(dev(synth.values(g, shape.B, shape.Hkv, 1, shape.D)))
        v_new.copy_(dev(synth.values(g, shape.B, shape.Hkv, 1, shape.D)))
        lens.fill_(shape.N + 1 + it)
        graph.replay()
        torch.cuda.synchronize()
        got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
        e_out, e_lse = _alloc(shape)
        step(e_out, e_lse, k_e, v_e, lens)             # eager, on its own copy of the caches
        torch.cuda.synchronize()
        np.testing.assert_array_equal(k_g.cpu().numpy(), k_e.cpu().numpy())
        np.testing.assert_array_equal(v_g.cpu().numpy(), v_e.cpu().numpy())
        np.testing.assert_array_equal(out.cpu().numpy(), e_out.cpu().numpy())
        np.testing.assert_array_equal(lse.cpu().numpy(), e_lse.cpu().numpy())
        if it == 3:                                    # and the last one against the oracle
            from helpers import oracle_view
            y = oracle_view(shape, dict(x, q=q.cpu().numpy(), k_idx=k_e.cpu().numpy(), v_idx=v_e.cpu().numpy()))
            ref = oracle.decode_attention(y["q"], y["lam"], y["cb_k"], y["cb_v"], y["k_idx"], y["v_idx"],
                                          np.full(shape.B, shape.N + 4))
            assert_decode_close(*got, *ref, what="graph replay vs oracle")


def test_read_probe_reads_and_writes_nothing():
    """The measurement aid: a plain read of a buffer whose size is not a multiple of anything nice;
    the sink keeps its value and the source is untouched."""
    src = torch.arange(3_000_017, dtype=torch.int32, device="cuda")
    before = src.clone()
    sink = torch.full((1,), 1234, dtype=torch.int32, device="cuda")
    view = src.view(torch.uint8)[: (src.numel() * 4) // 16 * 16 - 16]
    vb.vecinfer_read_probe(view, sink)
    vb.vecinfer_read_probe(src.view(torch.uint8)[:64], sink)        # fewer 16-byte pieces than workgroups
    torch.cuda.synchronize()
    assert int(sink.item()) == 1234 and torch.equal(src, before)
