#!/usr/bin/env python3
"""Benchmark of the fused VQ decode-attention hot path on one MI355X.

Workload (the long-context configuration the metric is quoted on): Llama-3.1-8B layer shape,
batch 1, 32 query / 8 KV heads, head dim 128, 196608 cached tokens, b2d4 codes for K and V.
One step = one decode step of one layer (vecinfer_decode_step): append the new token's key and
value codes (smooth + FWHT + nearest centroid) and run the fused VQ attention over the cache.
Steps rotate over several distinct layers (code caches, codebooks, smoothing factors) so that the index stream comes from HBM, not
from the 256 MB Infinity Cache.  Inputs are seeded and synthetic and are resident in HBM
before the timed region.

Prints ONE JSON line: `value` = index bytes per step / step time; `roofline.achieved` = index bytes /
average duration of the attention call, timed by its own event pairs; `cpu_baseline` = the float64
oracle on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "fused VQ decode-attn: compressed-KV GB/s (% HBM peak) + µs/step, 8B @196k"
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# Calls run untimed before anything is timed: the chip needs a few hundred back-to-back calls to
# reach its steady clock (a fresh process runs its first ~400 calls about 25 % slower).
PREWARM_CALLS = 1500


def measured_traffic(workload: str, tokens: int, v_tiled: int):
    """HBM bytes per attention launch from the committed rocprofv3 counter summaries
    (profiles/*_hbm_traffic.txt: FETCH_SIZE + WRITE_SIZE, each scaled by a copy kernel of known
    size).  A summary carries one line per workload it covers,
        traffic_bytes <workload> <tokens> <rows|tiled> <kernel> <fetch bytes> <write bytes>
    Returns (bytes, kernel, file name), or (None, None, reason) when no line matches."""
    folder = os.path.join(ROOT, "profiles")
    layout = "tiled" if v_tiled else "rows"
    try:
        names = sorted(n for n in os.listdir(folder) if n.endswith("_hbm_traffic.txt"))
    except OSError:
        return None, None, "no profiles folder"
    for name in names:
        with open(os.path.join(folder, name)) as f:
            for line in f:
                w = line.split()
                if len(w) == 7 and w[0] == "traffic_bytes" and w[1] == workload and int(w[2]) == tokens and w[3] == layout:
                    return float(w[5]) + float(w[6]), w[4], name
    return None, None, f"no rocprofv3 counter summary for {workload} at {tokens} tokens ({layout})"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="196k-b2d4",
                    choices=["196k-b2d4", "196k-b4d2", "32k", "batch32", "196k-d64", "196k-d64-d8", "196k-kd2vd4", "196k-d8b8", "196k-d8b12",
                             "196k-d4b12", "196k-kd4b10-vd8b12", "196k-kd8b12-vd8b8"])
    ap.add_argument("--tokens", type=int, default=0,
                    help="override the workload's cache length N (the 32k .. 196k ladder); a side measurement")
    ap.add_argument("--layers", type=int, default=0, help="distinct layer caches to rotate over (0 = auto)")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--variant", default="auto", choices=["auto", "lut", "mfma", "roles"])
    ap.add_argument("--v-layout", default="auto", choices=["auto", "rows", "tiled"],
                    help="physical layout of the value code cache: rows [n_cap, M_v], or tiles of 64 tokens "
                         "in the attention kernel's own order (cfg.v_tiled); auto = tiled where it applies "
                         "(8-bit codes on both sides, matrix-core kernel)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run 8 plain 256 MiB device copies first: a kernel of known HBM traffic "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    ap.add_argument("--residual", type=int, default=0,
                    help="keep this many most recent tokens in a full-precision fp16 window (at most 128) and "
                         "attend to them in the same call; the new token then goes into the window (a copy on "
                         "the caller's side), so the step has no append - a side measurement, not the metric")
    ap.add_argument("--separate-append", action="store_true",
                    help="append with vecinfer_append_kv and attend with vecinfer_decode_attention (two calls) "
                         "instead of the fused vecinfer_decode_step")
    ap.add_argument("--decode-only", action="store_true",
                    help="time the attention call alone (no append) - for profiling, not the metric")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only; --gpus must be 1 "
              "(the path shards by KV head, batch or sequence with one log-sum-exp merge; not built).", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2510_06175_amd import binding as vb
    from paper_2510_06175_amd import synth

    shape = {"196k-b2d4": synth.LLAMA8B_196K, "196k-b4d2": synth.LLAMA8B_196K_B4D2,
             "32k": synth.LLAMA8B_32K, "batch32": synth.LLAMA8B_BATCH32,
             "196k-d64": synth.HEADDIM64_196K, "196k-kd2vd4": synth.LLAMA8B_196K_KD2_VD4,
             "196k-d64-d8": synth.Shape(1, 32, 8, 64, 196608, 8, 8),      # head dim 64, 1-bit keys and values
             "196k-d8b8": synth.Shape(1, 32, 8, 128, 196608, 8, 8),       # 1 bit per element (d8b8)
             # codes wider than 8 bits, one shared codebook per KV head (side measurements, not the metric)
             "196k-d8b12": synth.LLAMA8B_196K_D8B12,
             "196k-d4b12": synth.Shape(1, 32, 8, 128, 196608, 4, 4, 12, 12),
             "196k-kd4b10-vd8b12": synth.Shape(1, 32, 8, 128, 196608, 4, 8, 10, 12),
             "196k-kd8b12-vd8b8": synth.Shape(1, 32, 8, 128, 196608, 8, 8, 12, 8)}[args.workload]
    if args.tokens:
        shape = synth.Shape(shape.B, shape.Hq, shape.Hkv, shape.D, args.tokens, shape.d_k, shape.d_v, shape.b_k, shape.b_v)
    variant = {"auto": vb.VARIANT_AUTO, "lut": vb.VARIANT_LUT, "mfma": vb.VARIANT_MFMA, "roles": vb.VARIANT_ROLES}[args.variant]
    can_tile = shape.b_k == 8 and shape.b_v == 8 and variant != vb.VARIANT_LUT and shape.N % 64 == 0 and shape.Mv >= 16
    if args.v_layout == "tiled" and not can_tile:
        print("bench.py: --v-layout tiled needs 8-bit codes on both sides, the matrix-core kernel and "
              "a cache length that is a multiple of 64", file=sys.stderr)
        return 2
    v_tiled = 1 if (args.v_layout == "tiled" or (args.v_layout == "auto" and can_tile)) else 0
    cfg = vb.Config(shape.D, shape.Hq, shape.Hkv, shape.d_k, shape.d_v, shape.b_k, shape.b_v, v_tiled)
    idx_bytes = shape.index_bytes()
    layers = args.layers or max(2, -(-768 * 2**20 // idx_bytes))   # working set >= 768 MB > Infinity Cache
    torch.cuda.set_device(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    # ---- inputs, resident in HBM
    x0 = synth.decode_inputs(shape, seed=4)
    # every layer has its own code cache, codebooks and smoothing factors (layer 0 = x0, which the
    # oracle leg also uses); the query is the same tensor for all
    q = dev(x0["q"])
    caches = [tuple(dev(x0[k]) for k in ("k_idx", "v_idx", "cb_k", "cb_v", "lam"))]
    if v_tiled:
        # the random bytes of layer 0's value cache are taken as a tiled cache; the oracle leg gets
        # the N x M_v code matrix they hold (codes are uniform random either way)
        rows = torch.empty_like(caches[0][1])
        vb.vecinfer_export_value_codes(cfg, caches[0][1], rows)
        torch.cuda.synchronize()
        x0["v_idx"] = rows.cpu().numpy()
        del rows
    for layer in range(1, layers):
        g = synth.rng(1000 + layer)
        caches.append((dev(synth.random_code_rows(g, shape.B, shape.Hkv, shape.N, shape.row_bytes_k)),
                       dev(synth.random_code_rows(g, shape.B, shape.Hkv, shape.N, shape.row_bytes_v)),
                       dev(synth.codebooks_for(g, shape.Hkv, shape.Mk, shape.d_k, shape.b_k)),
                       dev(synth.codebooks_for(g, shape.Hkv, shape.Mv, shape.d_v, shape.b_v)),
                       dev(synth.lognormal_lambda(g, shape.Hkv, shape.D))))
    g = synth.rng(77)
    new_k = dev(synth.values(g, shape.B, shape.Hkv, 1, shape.D))
    new_v = dev(synth.values(g, shape.B, shape.Hkv, 1, shape.D))
    ws = vb.new_workspace(cfg, shape.B, shape.N, args.splits)
    out = torch.empty((shape.B, shape.Hq, shape.D), dtype=torch.float16, device="cuda")
    lse = torch.empty((shape.B, shape.Hq), dtype=torch.float32, device="cuda")
    splits = args.splits or vb.vecinfer_decode_auto_splits(cfg, shape.B, shape.N)

    if args.residual:
        args.decode_only = True
        win = {k: dev(v) for k, v in synth.residual_window(shape, seed=78, r_cap=args.residual).items()}

    def attend(i):
        k_idx, v_idx, cb_k, cb_v, lam = caches[i % layers]
        if args.residual:
            vb.vecinfer_decode_attention_residual(cfg, q, lam, cb_k, cb_v, k_idx, v_idx, win["k_res"], win["v_res"],
                                                  ws, out, lse=lse, num_splits=args.splits, variant=variant)
            return
        vb.vecinfer_decode_attention(cfg, q, lam, cb_k, cb_v, k_idx, v_idx, ws, out, lse=lse,
                                     num_splits=args.splits, variant=variant)

    def step(i):
        if args.decode_only:
            attend(i)
            return
        k_idx, v_idx, cb_k, cb_v, lam = caches[i % layers]
        if args.separate_append:
            vb.vecinfer_append_kv(cfg, new_k, new_v, lam, cb_k, cb_v, k_idx, v_idx, pos0=shape.N - 1)
            attend(i)
        else:
            vb.vecinfer_decode_step(cfg, q, new_k, new_v, lam, cb_k, cb_v, k_idx, v_idx, ws, out, lse=lse,
                                    num_splits=args.splits, variant=variant)

    if args.traffic_probe:
        src = torch.empty(256 * 2**20, dtype=torch.uint8, device="cuda").random_(0, 256)
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- clock pre-conditioning (untimed, reported as prewarm_calls): the plain read probe and a
    # fixed count of calls of each kind that is timed below
    big = torch.empty(2**30, dtype=torch.uint8, device="cuda").random_(0, 256)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(3):
        vb.vecinfer_read_probe(big, sink)
    for i in range(PREWARM_CALLS):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: W warm-up steps, then exactly K steps between events on the launch stream
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    value = idx_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- dominant kernel (the attention call: attention kernel + split merge), no append: its
    # average duration over K back-to-back calls between two events on the launch stream, right
    # behind the step leg (the same clock state, and its own W warm-up calls), and the
    # spread from one event pair per call (a pair adds its own overhead to the call it brackets)
    # (at least 400 calls whatever K is: an average over a 20-call window of 0.6 ms carries the
    # ramp of its first launches, +-1 us per call)
    kern_calls = max(args.steps, 400)
    for i in range(max(args.warmup, 50)):
        attend(i)
    torch.cuda.synchronize()
    e0.record()
    for i in range(kern_calls):
        attend(i)
    e1.record()
    torch.cuda.synchronize()
    kern_avg_ms = e0.elapsed_time(e1) / kern_calls
    achieved = idx_bytes / (kern_avg_ms * 1e-3) / 1e9
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
             for _ in range(400)]
    for i, (a, b) in enumerate(pairs):
        a.record()
        attend(i)
        b.record()
    torch.cuda.synchronize()
    kern_ms = sorted(a.elapsed_time(b) for a, b in pairs)

    # ---- what a plain read reaches on this machine: vecinfer_read_probe (a kernel that only loads) over
    # one 1 GiB buffer, so that neither launch costs nor the Infinity Cache flatter or hurt it
    for _ in range(3):
        vb.vecinfer_read_probe(big, sink)
    torch.cuda.synchronize()
    probe_n = 20
    e0.record()
    for _ in range(probe_n):
        vb.vecinfer_read_probe(big, sink)
    e1.record()
    torch.cuda.synchronize()
    probe_gbs = big.numel() * probe_n / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del big
    traffic, traffic_kernel, traffic_src = (measured_traffic(args.workload, shape.N, v_tiled)
                                            if variant != vb.VARIANT_LUT else (None, None, "lookup-table variant: not profiled"))

    rec = {
        "metric": METRIC, "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "prewarm_calls": PREWARM_CALLS, "ms_per_step": round(ms_per_step, 6), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8 codes, f16 tables, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{'llama-3.1-8b' if shape.D == 128 else 'head-dim-64'} layer decode, B={shape.B}, Hq={shape.Hq}, Hkv={shape.Hkv}, "
                               f"D={shape.D}, N={shape.N}, K d{shape.d_k}b{shape.b_k} / V d{shape.d_v}b{shape.b_v}",
                   "step": f"attention over the code cache and a {args.residual}-token fp16 window" if args.residual
                   else "attention only" if args.decode_only
                   else "append 1 token (smooth+FWHT+VQ of k, VQ of v) + fused VQ attention, "
                        + ("two calls" if args.separate_append else "one call (vecinfer_decode_step)"),
                   "index_bytes_per_step": idx_bytes, "layer_caches_rotated": layers,
                   "value_code_layout": "tiles of 64 tokens" if v_tiled else "rows",
                   "num_splits": splits, "variant": args.variant,
                   "us_per_step": round(ms_per_step * 1e3, 3),
                   "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2)},
        # `kernel` is the call the events bracket: the attention kernel plus, with more than one split,
        # the merge kernel right behind it (rocprofv3 lists the two separately, see profiles/)
        "roofline": {"bound": "hbm", "kernel": "vecinfer_decode_attention",
                     "launches_per_call": [{vb.VARIANT_LUT: "decode_lut_kernel", vb.VARIANT_ROLES: "decode_roles_kernel"}.get(variant, "decode_mfma_kernel")]
                     + (["merge_kernel"] if splits > 1 else []),
                     "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_kernel": traffic_kernel, "traffic_source": traffic_src,
                     "algorithmic_bytes": idx_bytes, "kernel_us_avg": round(kern_avg_ms * 1e3, 3), "kernel_calls_timed": kern_calls,
                     "event_pair_us_median": round(kern_ms[len(kern_ms) // 2] * 1e3, 3),
                     "event_pair_us_min": round(kern_ms[0] * 1e3, 3),
                     "plain_read_probe_gbs": round(probe_gbs, 1),
                     "frac_of_plain_read_probe": round(achieved / probe_gbs, 4)},
    }

    # ---- the oracle (as it stands) on the host cores: the same attention step on layer cache 0,
    # repeated until about 10 s of wall time have passed (bounded sample of the same workload).
    # Its result also checks the kernel that was just timed: the attention call on layer cache 0
    # must agree with it to the parity bar of the tests, or no line is printed.
    if not args.no_cpu_baseline:
        import oracle
        attend(0)
        torch.cuda.synchronize()
        gpu_o, gpu_l = out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
        ox = dict(x0)
        for side, bits, M in (("k", shape.b_k, shape.Mk), ("v", shape.b_v, shape.Mv)):
            if bits != 8:       # the oracle takes a shared codebook as [Hkv, 1, C, d] and unpacked indices
                ox["cb_" + side] = x0["cb_" + side][:, None]
                ox[side + "_idx"] = oracle.unpack_codes(x0[side + "_idx"], bits, M)
        reps, t0 = 0, time.perf_counter()
        while True:
            ref_o, ref_l = oracle.decode_attention(ox["q"], ox["lam"], ox["cb_k"], ox["cb_v"], ox["k_idx"], ox["v_idx"])
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= 10.0 or reps >= 64:
                break
        if not args.residual:
            rel = float((np.abs(gpu_o - ref_o).max(axis=-1) / np.abs(ref_o).max(axis=-1)).max())
            l_err = float(np.abs(gpu_l - ref_l).max())
            rec["parity_vs_oracle"] = {"max_err_over_out_inf": round(rel, 6), "tolerance": 2e-3,
                                       "max_abs_err_lse": round(l_err, 6), "tolerance_lse": 1e-3}
            if not (rel <= 2e-3 and l_err <= 1e-3):
                print(f"bench.py: the timed kernel disagrees with the oracle (output {rel:.3e}, L {l_err:.3e}); "
                      "no result line", file=sys.stderr)
                return 3
        rec["cpu_baseline"] = {"value": round(idx_bytes * reps / dt / 1e9, 5), "unit": "GB/s",
                               "cores": oracle.num_threads(), "kind": "oracle", "seconds": round(dt, 3),
                               "sample": f"{reps} full attention steps of this workload over layer cache 0 "
                                         "(float64 explicit dequantize-then-attend, OpenMP across the 32 heads; "
                                         "the append is not included)"}
    print(json.dumps(rec))
    return 0


if __name__ == "__main__":
    sys.exit(main())
