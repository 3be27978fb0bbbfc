#!/usr/bin/env python3
"""Benchmark: RGAT layer forward+backward on one MI355X, edges/s.

One step = one pass of the whole hot path (rgnn_rgat_fwd + rgnn_rgat_bwd) over the
synthetic 1M-node / 200-relation / 10M-edge graph, inputs resident in HBM, graph index
built beforehand (the thesis also times the layer only, with preprocessing done before).
Prints ONE JSON line with the throughput, the roofline of the dominant kernel (timed live
with HIP events on the launch stream, through the library's profiling hooks) and the CPU
oracle timed on the host cores on the same inputs.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3


def algorithmic_work(name, E, N, P, Q, R, T, d, H, P1=0, bf16=False, layer="rgat"):
    """(bound, bytes, flops) one launch of kernel `name` must move / compute.  Gathered rows are
    counted once per reference (no cache reuse assumed); index and scalar traffic as listed in the
    comments below.  Row tensors are 4-byte elements, except in the
    bfloat16 workloads at width 128, where inputs and intermediate rows are 2-byte elements
    (results handed back to the caller stay fp32)."""
    half = bf16 and d == 128
    r32 = d * 4                       # an fp32 row
    row = d * 2 if half else r32      # an input / intermediate row
    wb = 2 if half else 4             # element size of a given weight
    # width 128: the backward typed linear is two kernels, "<label>" = dY W^T and "<label>.wgrad"
    # (bf16 rows: always; fp32 rows: wherever the rank-1 extras of single-head RGAT are not needed)
    split = d == 128 and (half or layer != "rgat" or H > 1)
    if split:
        rows = {"typed_linear": P, "pair_linear": P, "node_linear": N, "self_loop": N}
        key = name.split(".")[0]
        n = next((v for k, v in rows.items() if key.startswith(k)), None)
        if n is not None and (half or key.endswith("_bwd")):
            bound = "hbm" if half else "mfma"
            # one row in, one row out (or two rows in for the weight gradient), + the gather index
            segs = T if key.startswith("node_linear") else (1 if key.startswith("self_loop") else R)
            w2 = d * d * (4 if key.startswith("pair_linear") else wb)       # block-diagonal weights are fp32
            if name.endswith(".wgrad"):
                return (bound, n * (2 * row + 4) + segs * d * d * 4, 2.0 * n * d * d)
            out_row = r32 if key in ("node_linear_out", "node_linear_k_bwd", "node_linear_q_bwd", "node_linear_v_bwd") else row
            extra = r32 if half and key in ("node_linear_q_bwd", "node_linear_v_bwd") else 0   # accumulate into dX
            return (bound, n * (row + out_row + extra + 4) + segs * w2, 2.0 * n * d * d)
    w2 = d * d * 4
    # single-head RGAT up to width 64: the gradient row of a single-edge pair is not stored per pair; the
    # backward typed linear reads att_e * dOut[dst_e] through a row selector (one index per pair; ds_src[p] and
    # the scale come as one pair of floats per pair)
    sel = layer == "rgat" and H == 1 and d <= 64
    pair_fwd = ("mfma", P * (2 * row + 4) + R * w2, 2.0 * P * d * d)        # gathered row + stored row + pair_src
    pair_bwd = ("mfma", P * (3 * row + 4) + R * w2, 4.0 * P * d * d)        # dY row + gathered row + stored row
    node_fwd = ("mfma", N * (2 * row + 4) + T * w2, 2.0 * N * d * d)
    node_bwd = ("mfma", N * (3 * row + 4) + T * w2, 4.0 * N * d * d)
    out_dst = row if layer == "hgt" else r32                                  # HGT's Z / dQ are intermediates
    agg_dst = ("hbm", E * (row + 4 + 4 * H) + N * (out_dst + 8), 2.0 * E * d)  # row + in_pair + coefficient(s); out row + item
    agg_pair = ("hbm", E * (row + 8 + 4 * H) + P * (row + 8), 2.0 * E * d)    # row + out_epos + out_dst + coefficient(s)
    table = {
        # RGAT: + s_src per pair and head; backward also reads ds_src
        "typed_linear_fwd": ("mfma", pair_fwd[1] + (P * 4 * H if layer == "rgat" else 0), pair_fwd[2]),
        "typed_linear_bwd": ("mfma", pair_bwd[1] + (P * 4 if layer == "rgat" else 0) + (P * 8 if sel else 0), pair_bwd[2]),
        "self_loop_fwd": ("mfma", N * 3 * r32 + w2, 2.0 * N * d * d),         # X row + out row read and written
        "self_loop_bwd": ("mfma", N * 3 * r32 + w2, 4.0 * N * d * d),
        "aggregate_fwd": agg_dst,
        # the same sum edge by edge with atomic adds: + in_run and run_dst per edge, and the zero fill
        "aggregate_fwd_edge_parallel": ("hbm", agg_dst[1] + E * 8 + N * r32, 2.0 * E * d),
        # per edge: Hs row + in_pair + att + (att, dz) store; per node: dOut row + out row + item;
        # per single-edge pair (P1 of them): ds_src and its G row, or with the row selector att_e only
        "edge_dot_bwd": ("hbm", E * (row + 16) + N * (2 * row + 8) + P1 * ((4 if sel else row) + 4), 2.0 * E * d),
        # RGAT: only the E - P1 edges of the P - P1 pairs with several edges; coefficient = the (att, dz) pair;
        # with one head the walk also writes ds_src per pair.
        # RGCN: every edge; row + out_dst + coefficient
        # RGCN with bf16 rows: likewise only pairs with several edges (the typed-linear backward reads the
        # others' rows straight from the destinations' gradient rows)
        "aggregate_bwd_pair": ("hbm", (E - P1) * (row + 16) + (P - P1) * (row + 8 + (4 if H == 1 else 0)), 2.0 * (E - P1) * d) if layer == "rgat"
                              else ("hbm", (E - P1) * (row + 8) + (P - P1) * (row + 8), 2.0 * (E - P1) * d) if half
                              else ("hbm", E * (row + 8) + P * (row + 8), 2.0 * E * d),
        # per run: X row + relrun_idx + run_dst + ds_dst
        "dst_side_wgrad": ("hbm", Q * (row + 12), 2.0 * Q * d),
        # per pair: dXp row + srcpair_idx; per run (RGAT): ds_dst + run_rel; per node: result row + 2 ptrs
        "node_grad_sum": ("hbm", P * (row + 4) + (Q * 8 if layer == "rgat" else 0) + N * (out_dst + 8), 1.0 * P * d),
        # per edge: in_pair, in_run, s_src, s_dst, att write (reads of its own writes not counted)
        "edge_softmax": ("hbm", E * 20 + N * 8, 10.0 * E),
        "run_logit": ("hbm", Q * (row + 12), 2.0 * Q * d),
        # HGT
        "node_linear_k": node_fwd, "node_linear_q": node_fwd, "node_linear_v": node_fwd, "node_linear_out": node_fwd,
        "node_linear_k_bwd": node_bwd, "node_linear_q_bwd": node_bwd, "node_linear_v_bwd": node_bwd,
        "node_linear_out_bwd": node_bwd,
        "pair_linear_att": pair_fwd, "pair_linear_msg": pair_fwd,
        "pair_linear_att_bwd": pair_bwd, "pair_linear_msg_bwd": pair_bwd,
        "hgt_edge_logit": ("hbm", E * (row + 4 + 4 * H) + N * (row + 8), 2.0 * E * d),
        "hgt_edge_dot_bwd": ("hbm", E * (row + 4 + 8 * H) + N * (2 * row + 8), 2.0 * E * d),
        "hgt_softmax": ("hbm", E * H * 8 + N * 8, 10.0 * E * H),
        "aggregate_bwd_msg": agg_pair, "aggregate_bwd_key": agg_pair, "aggregate_bwd_query": agg_dst,
    }
    return table.get(name)


def make_layer(c, g, heads=0, flags=0):
    """-> (layer object, forward-only?) for workload dict c on graph g."""
    from paper_2412_04747_amd.harness import RgatLayer, RgcnLayer, HgtLayer
    d, dt = c["d_out"], c["dtype"]
    if c["layer"] == "rgat":
        L = RgatLayer(g, d, c["slope"], dtype=dt, heads=max(heads, 1), flags=flags)
        L.load(c["X"], c["W"], c["w_s"], c["w_t"], c["dOut"])
    elif c["layer"] == "rgcn":
        L = RgcnLayer(g, d, c["norm"], "none", False, dtype=dt)
        L.load(c["X"], c["W"], None, c["dOut"])
    else:
        L = HgtLayer(g, d, c["H"], with_mu=False, dtype=dt)
        L.load(c["X"], c["Wk"], c["Wq"], c["Wv"], c["Wo"], c["Watt"], c["Wmsg"], None, c["dOut"])
    return L


def run_oracle(c):
    """-> (dict of expected outputs, seconds forward, seconds backward)."""
    from oracle import layers as O
    N, s, t, r = c["N"], c["src"], c["dst"], c["rel"]
    t0 = time.time()
    if c["layer"] == "rgat" and c["H"] > 1:
        out = O.rgat_heads_fwd(N, s, t, r, c["X"], c["W"], c["w_s"], c["w_t"], c["H"], c["slope"])
        tf = time.time() - t0; t0 = time.time()
        want = O.rgat_heads_bwd(N, s, t, r, c["X"], c["W"], c["w_s"], c["w_t"], c["dOut"], c["H"], c["slope"])
    elif c["layer"] == "rgat":
        out = O.rgat_fwd(N, s, t, r, c["X"], c["W"], c["w_s"], c["w_t"], c["slope"])
        tf = time.time() - t0; t0 = time.time()
        want = O.rgat_bwd(N, s, t, r, c["X"], c["W"], c["w_s"], c["w_t"], c["dOut"], c["slope"])
    elif c["layer"] == "rgcn":
        out = O.rgcn_fwd(N, s, t, r, c["X"], c["W"], None, c["norm"], "none")
        tf = time.time() - t0; t0 = time.time()
        want = {} if c["cid"] == 1 else O.rgcn_bwd(N, s, t, r, c["X"], c["W"], None, c["dOut"], c["norm"], "none", out=out)
        want.pop("dW0", None)
    else:
        names = ("X", "Wk", "Wq", "Wv", "Wo", "Watt", "Wmsg")
        out = O.hgt_fwd(N, s, t, r, c["ntype"], *[c[k] for k in names], None)
        tf = time.time() - t0; t0 = time.time()
        want = O.hgt_bwd(N, s, t, r, c["ntype"], *[c[k] for k in names], None, c["dOut"])
        want.pop("dmu", None)
    tb = time.time() - t0
    want["out"] = out
    return want, tf, tb


def train_step_bench(args):
    """Two-layer RGAT model, full-graph training step (forward, NLL loss, backward, SGD), the
    protocol of the thesis' evaluation section; one JSON line like the layer benchmark."""
    import numpy as np
    import torch
    from paper_2412_04747_amd import synth, binding as B, autograd as A
    c = synth.config(args.config, args.scale)
    if c["layer"] != "rgat":
        sys.exit("bench.py --train: pick an RGAT workload (--config 2 or 3)")
    N, R, E, d = c["N"], c["R"], c["E"], c["d_out"]
    g = A.Graph(N, R, c["src"], c["dst"], c["rel"])
    torch.manual_seed(synth.SEED0)
    layers = [A.RgatConv(R, d, c["slope"]), A.RgatConv(R, d, c["slope"])]
    params = [q for l in layers for q in l.parameters()]
    X = torch.tensor(c["X"], dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(synth.SEED0)
    train = torch.as_tensor(rng.choice(N, max(N // 10, 1), replace=False), device="cuda")
    labels = torch.as_tensor(rng.integers(0, d, len(train)), device="cuda")
    opt = torch.optim.SGD(params, lr=1e-3)

    def step():
        opt.zero_grad(set_to_none=True)
        h = layers[1](g, torch.relu(layers[0](g, X)))
        loss = torch.nn.functional.nll_loss(torch.log_softmax(h[train], dim=1), labels)
        loss.backward()
        opt.step()
        return loss

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.rgnn_profile_start()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    rep = B.rgnn_profile_stop()
    lib_ms = sum(ms for _, ms in rep.values()) / args.steps
    print(f"[bench] train step {dt * 1e3 / args.steps:.3f} ms, of which {lib_ms:.3f} ms in the library's kernels; "
          f"last loss {loss.item():.4f}", file=sys.stderr, flush=True)
    print(json.dumps({
        "metric": "edges/sec for 2-layer RGAT training step (fwd + NLL loss + bwd + SGD)",
        "value": 2 * E * args.steps / dt, "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}] graph, two RGAT layers of width {d}, N={N}, R={R}, E={E}; "
                               "value counts every edge once per layer"},
        "library_kernel_ms_per_step": lib_ms}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3,
                    help="synthetic workload id 1..5 (default 3 = the headline RGAT graph the metric is quoted on)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only)")
    ap.add_argument("--no-oracle", action="store_true", help="skip the CPU oracle leg (no cpu_baseline, no parity)")
    ap.add_argument("--dtype", choices=("f32", "bf16"), default=None,
                    help="override the storage type of the workload's inputs (the values stay the same)")
    ap.add_argument("--heads", type=int, default=0, help="RGAT workloads: number of attention heads (default 1)")
    ap.add_argument("--edge-parallel", action="store_true",
                    help="single-head RGAT: forward aggregation edge by edge with atomic adds (comparison schedule)")
    ap.add_argument("--fwd-only", action="store_true",
                    help="time the forward call alone (inference: no saved buffer is kept)")
    ap.add_argument("--graph", action="store_true",
                    help="record one step into a HIP graph and time its replays (no per-kernel breakdown: the "
                         "timing events cannot be recorded into a graph)")
    ap.add_argument("--train", action="store_true",
                    help="time a full training step instead: two RGAT layers through the autograd front end, "
                         "log-softmax + NLL loss on 10%% of the nodes, SGD update (RGAT workloads only)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (--gpus 1); sharding over several GPUs is a design "
                 "note, not code.")

    import numpy as np
    import torch
    from paper_2412_04747_amd import synth, binding as B
    from paper_2412_04747_amd.harness import Graph

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.train:
        return train_step_bench(args)
    t0 = time.time()
    c = synth.config(args.config, args.scale)
    if args.dtype:
        if args.dtype == "bf16" and c["dtype"] != "bf16":
            for k, v in list(c.items()):
                if isinstance(v, np.ndarray) and v.dtype == np.float32:
                    c[k] = synth.round_to_bf16(v)
        c["dtype"] = args.dtype
    if args.heads > 1:
        if c["layer"] != "rgat":
            sys.exit("bench.py --heads: only the RGAT workloads take a head count")
        c["H"] = args.heads
    N, R, E, d, T, H = c["N"], c["R"], c["E"], c["d_out"], c["T"], c["H"]
    fwd_only = c["cid"] == 1 or args.fwd_only
    print(f"[bench] generated config {args.config} ({c['layer']}, {c['dtype']}): N={N} T={T} R={R} E={E} d={d} H={H} "
          f"in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    cpu = None
    want = None
    if not args.no_oracle:
        from oracle import layers as O
        want, t_f, t_b = run_oracle(c)
        if fwd_only:
            t_b = 0.0
        cpu = {"value": E / (t_f + t_b), "unit": "edges/s", "cores": O.num_threads(), "kind": "oracle",
               "sample": f"full workload, 1 repetition (fwd {t_f:.2f}s + bwd {t_b:.2f}s)"}
        print(f"[bench] oracle fwd {t_f:.2f}s bwd {t_b:.2f}s on {O.num_threads()} threads", file=sys.stderr, flush=True)

    t0 = time.time()
    g = Graph(N, R, c["src"], c["dst"], c["rel"], c.get("ntype") if T > 1 else None, T,
              c.get("rel_src_ntype"), c.get("rel_dst_ntype"))
    P, Q = g.P, g.Q
    P1 = int(g.info.num_single_pairs) if c["layer"] in ("rgat", "rgcn") else 0
    print(f"[bench] graph index built in {time.time() - t0:.1f}s: P/E={P / E:.3f} Q/E={Q / E:.3f} "
          f"max in-degree {g.info.max_in_degree} index {g.info.index_bytes / 2**20:.0f} MiB", file=sys.stderr, flush=True)
    if args.edge_parallel and (c["layer"] != "rgat" or args.heads > 1):
        sys.exit("bench.py --edge-parallel: single-head RGAT workloads only")
    L = make_layer(c, g, args.heads, 1 if args.edge_parallel else 0)

    def step():
        L.fwd()
        if not fwd_only:
            L.bwd()

    # One plain 1 GiB device-to-device copy before the timed region: a kernel of known size
    # against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are calibrated.
    cal = torch.empty(2, 1 << 28, dtype=torch.float32, device="cuda")
    cal[0].fill_(1.0)
    cal[1].copy_(cal[0])
    torch.cuda.synchronize()
    del cal

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        hip_graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            side.synchronize()
            with torch.cuda.graph(hip_graph, stream=side):
                step()
        torch.cuda.synchronize()
        for _ in range(args.warmup):
            hip_graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            hip_graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        print(json.dumps({
            "metric": f"edges/sec for {c['layer'].upper()} layer {'fwd' if fwd_only else 'fwd+bwd'} (HIP graph replay)",
            "value": E * args.steps / dt, "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": dt * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16" if c["dtype"] == "bf16" else "f32", "data": "synthetic",
            "config": {"workload": f"configs[{args.config - 1}]: {c['layer'].upper()}, {c['dtype']} inputs, N={N}, R={R}, E={E}, d={d}"},
            "cpu_baseline": cpu}), flush=True)
        return
    # untimed clean pass, to show what the profiling events cost
    tc = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    clean_ms = (time.perf_counter() - tc) * 1e3 / args.steps

    B.rgnn_profile_start()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    rep = B.rgnn_profile_stop()
    ms_per_step = dt * 1e3 / args.steps

    parity = None
    if want is not None:
        parity = {}
        got = dict(out=L.out, **({} if fwd_only else L.grads()))
        for k, v in got.items():
            if k not in want:
                continue
            a = v.cpu().numpy().astype(np.float64)
            parity[k] = float(np.abs(a - want[k]).max() / max(np.abs(want[k]).max(), 1e-30))
        print(f"[bench] max relative error vs oracle: {parity}", file=sys.stderr, flush=True)

    kernels = []
    for name, (n, ms) in rep.items():
        avg_ms = ms / n
        w = algorithmic_work(name, E, N, P, Q, R, T, d, H, P1, c["dtype"] == "bf16", c["layer"])
        row = {"name": name, "launches_per_step": n / args.steps, "avg_ms": avg_ms, "ms_per_step": ms / args.steps}
        if w:
            row["GBps"] = w[1] / avg_ms / 1e6
            row["TFLOPs"] = w[2] / avg_ms / 1e9
            row["bound"] = w[0]
        kernels.append(row)
    kernels.sort(key=lambda r: -r["ms_per_step"])
    for r in kernels:
        print("[bench] {name:28s} {ms_per_step:8.3f} ms/step  avg {avg_ms:8.3f} ms  {gb:>9s} GB/s {tf:>8s} TF/s".format(
            gb=f"{r['GBps']:.0f}" if "GBps" in r else "-", tf=f"{r['TFLOPs']:.1f}" if "TFLOPs" in r else "-", **r),
            file=sys.stderr, flush=True)
    dom = kernels[0]
    w = algorithmic_work(dom["name"], E, N, P, Q, R, T, d, H, P1, c["dtype"] == "bf16", c["layer"])
    if w and w[0] == "mfma":
        roof = {"kernel": dom["name"], "bound": "mfma", "achieved": dom["TFLOPs"], "peak": FP32_MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": dom["TFLOPs"] / FP32_MFMA_PEAK_TFLOPS, "traffic": None}
    else:
        gb = dom.get("GBps", 0.0)
        roof = {"kernel": dom["name"], "bound": "hbm", "achieved": gb, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gb / HBM_PEAK_GBS, "traffic": None}
    # HBM bytes per launch from rocprofv3 counters (two --pmc runs of this same command, calibrated
    # against the 1 GiB copy above); only valid for the full-size default workload.
    tsv = os.path.join(ROOT, "profiles", "rgat_c3_hbm_traffic_per_label.txt")
    if args.config == 3 and args.scale == 1.0 and os.path.exists(tsv):
        for ln in open(tsv):
            f = ln.rstrip("\n").split("\t")
            if not ln.startswith("#") and f[0] == dom["name"]:
                roof["traffic"] = float(f[1]) + float(f[2])
    roof["avg_ms"] = dom["avg_ms"]
    roof["algorithmic_bytes"] = w[1] if w else None
    # the same for the forward edge-traversal kernel (weighted gather-sum over the destination-major CSR),
    # the HBM-bound counterpart of the typed linear
    trav = next((k for k in kernels if k["name"] == "aggregate_fwd" and "GBps" in k), None)
    roof_trav = None
    if trav:
        roof_trav = {"kernel": "aggregate_fwd", "bound": "hbm", "achieved": trav["GBps"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": trav["GBps"] / HBM_PEAK_GBS, "traffic": None, "avg_ms": trav["avg_ms"]}
        if args.config == 3 and args.scale == 1.0 and os.path.exists(tsv):
            for ln in open(tsv):
                f = ln.rstrip("\n").split("\t")
                if not ln.startswith("#") and f[0] == "aggregate_fwd":
                    roof_trav["traffic"] = float(f[1]) + float(f[2])

    line = {
        "metric": f"edges/sec for {c['layer'].upper()} layer {'fwd' if fwd_only else 'fwd+bwd'}",
        "value": E * args.steps / dt, "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        # the arithmetic type of the path: fp32 throughout, or bf16 storage / bf16 matrix-core operands with
        # fp32 accumulation for the bfloat16 workloads
        "dtype": "bf16" if c["dtype"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}]: {c['layer'].upper()} {'fwd' if fwd_only else 'fwd+bwd'}, "
                               f"{c['dtype']} inputs, N={N}, T={T}, R={R}, E={E}, d={d}, H={H}"
                               + ("" if args.scale == 1.0 else f" (scale {args.scale})"),
                   "P_over_E": P / E, "Q_over_E": Q / E, "max_in_degree": int(g.info.max_in_degree)},
        "roofline": roof,
        "roofline_traversal": roof_trav,
        "cpu_baseline": cpu,
        "ms_per_step_without_profiling_events": clean_ms,
        "parity_max_rel_err": parity,
        "kernels": kernels,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
