"""Replay of a dumped decode case (``--load-case PREFIX``, written by ``--dump-case``): the GPU library
against the oracle on exactly the stored arrays and call arguments.  Skipped when no case is given.
The dump / load round trip itself is checked on the host."""
import numpy as np
import pytest

from paper_2510_06175_amd import synth

import helpers


def test_dump_and_load_round_trip(tmp_path):
    shape = synth.Shape(2, 8, 2, 128, 70, 4, 4)
    x = synth.decode_inputs(shape, seed=3)
    args = {"seq_lens": [70, 9], "N": 70, "num_splits": 3, "variant": 2, "v_tiled": 0}
    prefix = str(tmp_path / "sub" / "case")
    helpers.dump_case(prefix, "decode", shape, {k: x[k] for k in helpers.DECODE_KEYS}, args)
    kind, shape2, arrays, args2 = helpers.load_case(prefix)
    assert kind == "decode" and shape2 == shape and args2 == args
    assert list(arrays) == list(helpers.DECODE_KEYS)
    for k in helpers.DECODE_KEYS:
        assert arrays[k].dtype == x[k].dtype
        np.testing.assert_array_equal(arrays[k], x[k])


@pytest.mark.gpu
def test_replay_dumped_case(request):
    prefix = request.config.getoption("--load-case")
    if not prefix:
        pytest.skip("no --load-case given")
    import oracle
    kind, shape, x, args = helpers.load_case(prefix)
    assert kind == "decode"
    N = args["N"] if args["N"] is not None else x["k_idx"].shape[2]
    lens = None if args["seq_lens"] is None else np.asarray(args["seq_lens"])
    got = helpers.gpu_decode(shape, x, seq_lens=lens, N=N, num_splits=args["num_splits"], variant=args["variant"],
                             v_tiled=args["v_tiled"])
    ox = helpers.oracle_view(shape, x)
    v_idx = ox["v_idx"]
    if args["v_tiled"]:
        pytest.skip("tiled value codes: export them to rows with vecinfer_export_value_codes before replaying")
    keep = np.arange(x["q"].shape[0]) if lens is None else np.nonzero(lens > 0)[0]
    ref = oracle.decode_attention(ox["q"][keep], ox["lam"], ox["cb_k"], ox["cb_v"], ox["k_idx"][keep][:, :, :N],
                                  v_idx[keep][:, :, :N], None if lens is None else lens[keep])
    helpers.assert_decode_close(got[0][keep], got[1][keep], *ref, what=f"replay of {prefix}")
