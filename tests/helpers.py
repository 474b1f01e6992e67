"""Helpers of the GPU parity tests: run the library on numpy inputs, compare with the oracle.

A failing seeded case can be kept and replayed: with ``pytest --dump-case DIR`` the inputs of the
last decode call of every failing test are written as ``DIR/<test>.bin`` (the arrays, flat, one
after the other) plus ``DIR/<test>.json`` (names, dtypes, shapes, byte offsets, the shape and call
arguments); ``pytest tests/test_replay_case.py --load-case DIR/<test>`` runs that case alone, GPU
against oracle.  The method's persistent state is just these arrays (smoothing factors, codebooks,
code caches, query)."""
import json
import os

import numpy as np
import torch

from paper_2510_06175_amd import binding as vb

# Tolerances of the parity bar:
#   output  max |err| <= 2e-3 * ||out||_inf per (batch, head) row (fp16 output, fp32 accumulation)
#   L       |err| <= 1e-3 (scores and their log-sum-exp are O(10); fp32 rounding of a sum of
#           D terms plus the exp2/log2 units stays orders below this)
OUT_RTOL_INF = 2e-3
LSE_ATOL = 1e-3
NEAR_TIE = 1e-6     # relative distance gap under which an index mismatch is a logged near-tie


def cfg_of(shape, v_tiled=0):
    return vb.Config(shape.D, shape.Hq, shape.Hkv, shape.d_k, shape.d_v, shape.b_k, shape.b_v, v_tiled)


def tile_value_codes(rows):
    """Value codes [B, Hkv, n_cap, M] (n_cap a multiple of 64) -> the tiled layout of the C header
    ("Tiled value codes"), written out from its formula: byte of (t, m) at
    (t/64) 64M + (j/16) 1024 + ((i%4) 16 + m/R) 16 + j%16 with i = t % 64, R = M/16,
    j = ((i/16) 4 + (i%16)/4) R + m%R."""
    rows = np.asarray(rows)
    B, H, n_cap, M = rows.shape
    assert n_cap % 64 == 0 and M % 16 == 0
    R = M // 16
    t = np.arange(n_cap)[:, None]
    m = np.arange(M)[None, :]
    i = t % 64
    j = ((i // 16) * 4 + (i % 16) // 4) * R + m % R
    off = (t // 64) * 64 * M + (j // 16) * 1024 + ((i % 4) * 16 + m // R) * 16 + j % 16
    out = np.empty((B, H, n_cap * M), dtype=rows.dtype)
    out[:, :, off.reshape(-1)] = rows.reshape(B, H, -1)
    return out.reshape(B, H, n_cap, M)


def oracle_view(shape, x):
    """GPU-layout inputs as the oracle takes them: codebooks [Hkv, Mcb, C, d] (Mcb = 1 for the shared
    table of codes wider than 8 bits) and one unpacked index per sub-vector (uint16 when packed)."""
    import oracle
    y = dict(x)
    for side, bits, M in (("k", shape.b_k, shape.Mk), ("v", shape.b_v, shape.Mv)):
        if bits != 8:
            y["cb_" + side] = np.asarray(x["cb_" + side])[:, None]
            if side + "_idx" in x:
                y[side + "_idx"] = oracle.unpack_codes(np.asarray(x[side + "_idx"]), bits, M)
    return y


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


DECODE_KEYS = ("q", "lam", "cb_k", "cb_v", "k_idx", "v_idx")
last_case = None          # (kind, shape, arrays, call arguments) of the most recent decode call


def dump_case(prefix, kind, shape, arrays, args):
    """Write a case as prefix.bin (flat arrays) + prefix.json (header)."""
    os.makedirs(os.path.dirname(os.path.abspath(prefix)), exist_ok=True)
    import dataclasses
    header = {"kind": kind, "shape": list(dataclasses.astuple(shape)), "args": args, "arrays": []}
    off = 0
    with open(prefix + ".bin", "wb") as f:
        for name, a in arrays.items():
            a = np.ascontiguousarray(a.cpu().numpy() if isinstance(a, torch.Tensor) else a)
            f.write(a.tobytes())
            header["arrays"].append({"name": name, "dtype": str(a.dtype), "shape": list(a.shape), "offset": off,
                                     "nbytes": a.nbytes})
            off += a.nbytes
    with open(prefix + ".json", "w") as f:
        json.dump(header, f, indent=1)


def load_case(prefix):
    """-> (kind, synth.Shape, {name: numpy array}, call arguments) of a dumped case."""
    from paper_2510_06175_amd import synth
    with open(prefix + ".json") as f:
        header = json.load(f)
    blob = np.fromfile(prefix + ".bin", dtype=np.uint8)
    arrays = {}
    for e in header["arrays"]:
        raw = blob[e["offset"]:e["offset"] + e["nbytes"]]
        arrays[e["name"]] = raw.view(np.dtype(e["dtype"])).reshape(e["shape"]).copy()
    return header["kind"], synth.Shape(*header["shape"]), arrays, header["args"]


def gpu_decode(shape, x, seq_lens=None, N=None, num_splits=0, variant=vb.VARIANT_AUTO, ws=None, want_lse=True,
               v_tiled=0):
    """x: dict of numpy arrays (q, lam, cb_k, cb_v, k_idx, v_idx) -> (out fp16 as f64, lse f64)."""
    global last_case
    last_case = ("decode", shape, {k: x[k] for k in DECODE_KEYS},
                 {"seq_lens": None if seq_lens is None else [int(v) for v in np.asarray(seq_lens)],
                  "N": None if N is None else int(N), "num_splits": int(num_splits), "variant": int(variant),
                  "v_tiled": int(v_tiled)})
    cfg = cfg_of(shape, v_tiled)
    t = {k: (v if isinstance(v, torch.Tensor) else dev(v)) for k, v in x.items()
         if k in ("q", "lam", "cb_k", "cb_v", "k_idx", "v_idx")}
    B = t["q"].shape[0]
    n_cap = t["k_idx"].shape[2]
    N = n_cap if N is None else N
    if ws is None:
        ws = vb.new_workspace(cfg, B, N, num_splits)
    out = torch.full((B, shape.Hq, shape.D), float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full((B, shape.Hq), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    sl = None if seq_lens is None else torch.as_tensor(np.asarray(seq_lens), dtype=torch.int32).cuda()
    vb.vecinfer_decode_attention(cfg, t["q"], t["lam"], t["cb_k"], t["cb_v"], t["k_idx"], t["v_idx"], ws, out,
                                 lse=lse, seq_lens=sl, N=N, num_splits=num_splits, variant=variant)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64), (lse.cpu().numpy().astype(np.float64) if want_lse else None)


def gpu_decode_residual(shape, x, seq_lens=None, res_lens=None, N=None, R=None, num_splits=0,
                        variant=vb.VARIANT_AUTO):
    """As gpu_decode, plus the fp16 window x["k_res"], x["v_res"] [B, Hkv, r_cap, D]."""
    cfg = cfg_of(shape)
    t = {k: dev(v) for k, v in x.items() if k in ("q", "lam", "cb_k", "cb_v", "k_idx", "v_idx", "k_res", "v_res")}
    B = t["q"].shape[0]
    N = t["k_idx"].shape[2] if N is None else N
    ws = vb.new_workspace(cfg, B, N, num_splits)
    out = torch.full((B, shape.Hq, shape.D), float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full((B, shape.Hq), float("nan"), dtype=torch.float32, device="cuda")
    as_i32 = lambda a: None if a is None else torch.as_tensor(np.asarray(a), dtype=torch.int32).cuda()
    vb.vecinfer_decode_attention_residual(cfg, t["q"], t["lam"], t["cb_k"], t["cb_v"], t["k_idx"], t["v_idx"],
                                          t["k_res"], t["v_res"], ws, out, lse=lse, seq_lens=as_i32(seq_lens),
                                          res_lens=as_i32(res_lens), N=N, R=R, num_splits=num_splits,
                                          variant=variant)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


def assert_decode_close(got_out, got_lse, ref_out, ref_lse, what=""):
    B, Hq, _ = ref_out.shape
    worst = 0.0
    for b in range(B):
        for h in range(Hq):
            scale = np.abs(ref_out[b, h]).max()
            err = np.abs(got_out[b, h] - ref_out[b, h]).max()
            assert np.isfinite(got_out[b, h]).all(), f"{what}: non-finite output at b={b} h={h}"
            assert err <= OUT_RTOL_INF * scale, (
                f"{what}: b={b} h={h} max|err|={err:.3e} > {OUT_RTOL_INF}*{scale:.3e}")
            worst = max(worst, err / scale if scale > 0 else 0.0)
    if got_lse is not None:
        d = np.abs(got_lse - ref_lse).max()
        assert d <= LSE_ATOL, f"{what}: |L err|={d:.3e}"
    return worst


def gpu_encode(shape, k=None, lam=None, cb_k=None, v=None, cb_v=None, pos0=0, n_cap=None, v_tiled=0):
    """Encode keys and/or values on the GPU; returns uint8 numpy arrays [B, Hkv, n_cap, row bytes]."""
    cfg = cfg_of(shape, v_tiled)
    res = []
    if k is not None:
        B, Hkv, T, D = k.shape
        cap = T + pos0 if n_cap is None else n_cap
        idx = torch.full((B, Hkv, cap, shape.row_bytes_k), 0xEE, dtype=torch.uint8, device="cuda")
        vb.vecinfer_encode_keys(cfg, dev(k), dev(lam), dev(cb_k), idx, pos0=pos0)
        res.append(idx)
    if v is not None:
        B, Hkv, T, D = v.shape
        cap = T + pos0 if n_cap is None else n_cap
        idx = torch.full((B, Hkv, cap, shape.row_bytes_v), 0xEE, dtype=torch.uint8, device="cuda")
        vb.vecinfer_encode_values(cfg, dev(v), dev(cb_v), idx, pos0=pos0)
        res.append(idx)
    torch.cuda.synchronize()
    return [r.cpu().numpy() for r in res]


def assert_indices_match(got, ref, gap, what=""):
    """Bit-exact except where the oracle's own best/second-best relative gap is below NEAR_TIE."""
    diff = got != ref
    n_diff = int(diff.sum())
    if n_diff:
        bad = diff & ~(gap < NEAR_TIE)
        print(f"[near-tie log] {what}: {n_diff} of {diff.size} indices differ; "
              f"max oracle gap among them {gap[diff].max():.3e}")
        assert not bad.any(), (f"{what}: {int(bad.sum())} index mismatches with relative gap >= {NEAR_TIE} "
                               f"(worst {gap[bad].max():.3e})")
    return n_diff
