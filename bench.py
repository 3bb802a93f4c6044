"""Throughput of the state encoder + heads on one MI355X, with roofline and CPU-oracle baseline.

One step = one pass of the whole path over one packed synthetic meta-batch that is already
resident in HBM: sum of incoming edge attributes, embed MLP, R x (edge MLP + per-receiver sum,
node MLP), per-graph readout, policy/value heads (xrl_encode + xrl_policy_value) and, for the
update minibatch (configuration 5, the default) or with --backward, the backward pass through
heads and encoder (xrl_policy_value_backward + xrl_encode_backward). Prints ONE JSON line.

Every step is bracketed by HIP events on the library's stream (which is torch's current stream);
`value` uses the median step, `ms_per_step_mean` is the host clock over all K steps.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch;
# summaries under profiles/), each scaled by the same counter's reading for a 1 GiB device copy
# (factors 2.000 and 1.000). An entry is valid only for the kernel sources it was taken with: the
# hash covers the files the kernel is built from (comments and blank space apart); otherwise null.
TRAFFIC = {
    # configuration 2 (profiles/forward_config2_bf16_hbm_traffic.md): persistent forward kernels, weights in LDS
    (2, "bf16", "edge"): dict(sources=("mma.hip.h", "mlp2.hip.h", "mlp2p.hip.h"), sha256_16="c1095d7066032095",
                              bytes_per_launch=(11154.7 * 2.000 + 11599.5 * 1.000) * 1024),
    (2, "bf16", "node"): dict(sources=("mma.hip.h", "mlp2.hip.h", "mlp2p.hip.h"), sha256_16="c1095d7066032095",
                              bytes_per_launch=(15508.5 * 2.000 + 18218.2 * 1.000) * 1024),
    # configuration 4 (profiles/forward_config4_bf16_kernel_stats_and_traffic.md): register-stationary forward kernels
    (4, "bf16", "edge"): dict(sources=("mma.hip.h", "mlp2.hip.h", "mlp2r.hip.h"), sha256_16="b61a512bcdbfb016",
                              bytes_per_launch=(89442.7 * 2.000 + 70572.0 * 1.000) * 1024),
    (4, "bf16", "node"): dict(sources=("mma.hip.h", "mlp2.hip.h", "mlp2r.hip.h"), sha256_16="b61a512bcdbfb016",
                              bytes_per_launch=(118742.4 * 2.000 + 162434.5 * 1.000) * 1024),
    # configuration 5 (profiles/step_config5_bf16_hbm_traffic.md): backward through the node / edge MLP
    (5, "bf16", "bwd_node"): dict(sources=("mma.hip.h", "mlp2_bwd.hip.h", "mlp2_bwdz.hip.h"), sha256_16="4137d3e1b408b425",
                                  # mean of the five launches: four with dz2 given by the gradient gather, the topmost round's
                                  bytes_per_launch=(0.8 * (4635006.5 * 2.000 + 20977475.7 * 1.000) +
                                                    0.2 * (947049.9 * 2.000 + 29040546.5 * 1.000)) * 1024),
    (5, "bf16", "bwd_edge"): dict(sources=("mma.hip.h", "mlp2_bwd.hip.h", "mlp2_bwdz.hip.h"), sha256_16="4137d3e1b408b425",
                                  bytes_per_launch=(3545704.0 * 2.000 + 31035381.9 * 1.000) * 1024),
}


def source_hash(files):
    import hashlib
    h = hashlib.sha256()
    for f in files:                               # the code without its comments and blank space
        with open(os.path.join(ROOT, "paper_2304_14698_amd", "csrc", f), "r") as fh:
            for ln in fh:
                ln = ln.split("//")[0].strip()
                if ln:
                    h.update(ln.encode() + b"\n")
    return h.hexdigest()[:16]


def measured_traffic(config, precision, kernel):
    t = TRAFFIC.get((config, precision, kernel))
    if t is None or source_hash(t["sources"]) != t["sha256_16"]:
        return None
    return t["bytes_per_launch"]


def oracle_model(model):
    from oracle import xrl_oracle as O
    return O.default_model(**{k: model[k] for k in ("n_op_types", "n_node_dense", "d_edge", "d_global",
                                                    "hidden", "rounds", "mlp_layers", "head_hidden", "readout")})


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def oracle_baseline_forward(model, state, w, budget_s):
    """The float64 oracle's forward over whole graphs of the same meta-batch, for budget_s seconds."""
    import numpy as np
    from oracle import xrl_oracle as O
    om = oracle_model(model)
    G = len(state["graph_node_ptr"]) - 1
    t0 = time.perf_counter()
    done, embs = 0, []
    for g in range(G):
        embs.append(O.encode(om, w, state, graphs=[g])[0])
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    if done == G:
        O.policy_value(om, w, np.stack(embs), state)
    dt = time.perf_counter() - t0
    return dict(value=done / dt, unit="graphs/s", cores=host_threads(), kind="oracle",
                sample=f"forward of {done} of {G} graphs of the same meta-batch, float64 numpy, {dt:.1f} s")


def oracle_baseline_update(model, state, w, up, n_states):
    """Forward + backward of the float64 oracle on the n_states whole states of the meta-batch with
    the fewest slots (all their graphs). The encoder's reverse mode evaluates the forward itself,
    so the timed work is one forward and one backward per graph: heads forward, heads backward,
    then forward + backward of the encoder (the embeddings the heads need come from an untimed
    first encode)."""
    import numpy as np
    import synth
    from oracle import xrl_oracle as O
    om = oracle_model(model)
    sgp = np.asarray(state["state_graph_ptr"])
    order = np.argsort(np.diff(sgp), kind="stable")[:n_states]
    order = np.sort(order)
    sub = synth.state_subset(state, order)
    gsel = np.concatenate([np.arange(sgp[s], sgp[s + 1]) for s in order])
    emb = O.encode(om, w, sub)                                  # untimed (see above)
    t0 = time.perf_counter()
    O.policy_value(om, w, emb, sub)
    demb, _ = O.policy_value_backward(om, w, emb, sub, up[0][gsel], up[1][order], up[2][order])
    O.encode_backward(om, w, sub, demb)
    dt = time.perf_counter() - t0
    Gs = len(gsel)
    return dict(value=Gs / dt, unit="graphs/s", cores=host_threads(), kind="oracle",
                sample=f"forward + backward of states {order.tolist()} ({Gs} graphs, "
                       f"{int(sub['node_op'].shape[0])} nodes: the {n_states} whole states of the same "
                       f"meta-batch with the fewest slots), float64 numpy, {dt:.1f} s")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 20 for configuration 5, else 200)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps first (default 5, or 20 below configuration 5)")
    ap.add_argument("--config", type=int, default=5,
                    help="synthetic configuration; 5 = the update minibatch, the largest that fits one GPU (default)")
    ap.add_argument("--precision", default=None, help="fp32 | bf16 (default: the configuration's)")
    ap.add_argument("--states", type=int, default=None, help="override the number of states")
    ap.add_argument("--round-kind", default="mlp", choices=["mlp", "gat"],
                    help="message-passing layers: edge/node MLPs (measured path) or graph attention")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-seconds", type=float, default=20.0,
                    help="CPU time given to the oracle's forward for the cpu_baseline figure (forward-only steps)")
    ap.add_argument("--cpu-baseline-states", type=int, default=4,
                    help="whole states the oracle runs forward + backward on (steps with the backward pass)")
    ap.add_argument("--no-segment-sum", action="store_true", help="skip the standalone [E, H] segment-sum timing")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one 1 GiB device-to-device copy (a kernel of known HBM traffic, the "
                         "reference that rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled by)")
    ap.add_argument("--peaks", action="store_true",
                    help="also measure the machine's own MFMA and copy rates (reported as measured_peaks)")
    ap.add_argument("--edit-pack", action="store_true",
                    help="also time packing + upload of a configuration-2-shaped state (12 transformer blocks, 128 "
                         "candidates) given as whole graphs and given as edits of the current graph (edit_pack)")
    ap.add_argument("--backward", action="store_true",
                    help="a step also runs both backward calls (always on for configuration 5)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if args.steps is None:
        args.steps = 20 if args.config == 5 else 200
    if args.warmup is None:
        args.warmup = 5 if args.config == 5 else 20

    import numpy as np
    import torch
    import paper_2304_14698_amd as xrl
    import synth
    xrl.load_library()
    assert torch.cuda.is_available(), "bench.py needs the GPU"

    model, state = synth.make_config(args.config, n_states=args.states)
    if args.precision:
        model["precision"] = args.precision
    model["round_kind"] = args.round_kind
    rng = np.random.Generator(np.random.PCG64(synth.BASE_SEED))
    w = synth.init_weights(rng, xrl.weight_layout(model), bias_range=0.1)
    enc = xrl.Encoder(model, w)
    t_pack = time.perf_counter()
    batch = enc.pack(state)                       # pack + upload happen before the timed region
    torch.cuda.synchronize()
    t_pack = time.perf_counter() - t_pack
    S, G, N, E = batch.S, batch.G, batch.N, batch.E
    H, R, De = model["hidden"], model["rounds"], model["d_edge"]
    Dd = model["n_node_dense"]
    emb = torch.empty((G, H), dtype=torch.float32, device="cuda")
    outs = dict(logp=torch.empty(G, device="cuda"), value=torch.empty(S, device="cuda"),
                entropy=torch.empty(S, device="cuda"), action=torch.empty(S, dtype=torch.int32, device="cuda"),
                logit=torch.empty(G, device="cuda"))

    backward = args.backward or args.config == 5
    up_host = None
    if backward:
        grng = np.random.Generator(np.random.PCG64(synth.BASE_SEED + 7))
        up_host = synth.upstream_grads(grng, G, S)
        up = [torch.from_numpy(np.ascontiguousarray(x)).cuda() for x in up_host]
        dw = torch.zeros(enc.n_weights, dtype=torch.float32, device="cuda")

    def step():
        enc.encode(batch, save_for_backward=backward, out=emb)
        enc.policy_value(batch, emb, out=outs)
        if backward:
            demb = enc.policy_value_backward(batch, emb, up[0], up[1], up[2], dw)
            enc.encode_backward(batch, demb, dw)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b_ in ev:
        a.record()
        step()
        b_.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = sorted(a.elapsed_time(b_) for a, b_ in ev)
    ms = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])
    ms_mean = dt / args.steps * 1e3

    # every launch group timed with HIP events on the library's stream over the same number of steps
    enc.set_timing(True)
    for _ in range(args.steps):
        step()
    kern = {}
    names = ("embed", "edge", "edge_fixup", "node", "gat_linear", "gat_aggregate", "pool", "readout", "heads", "resident")
    if backward:
        names += ("bwd_edge", "bwd_node", "bwd_embed", "wgrad_edge", "wgrad_node", "wgrad_embed", "grad_gather", "gat_bwd")
    for k in names:
        tot, n = enc.read_timing(k)
        kern[k] = dict(avg_us=(tot / n * 1e3 if n else 0.0), launches_per_step=n / args.steps)
    enc.set_timing(False)

    bf16 = model["precision"] == "bf16"
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS
    b = 2 if bf16 else 4
    hv = batch.host_view()
    n_recv = int((np.diff(hv["in_ptr"]) > 0).sum())
    n_tiles = len(hv["tile_ptr"]) - 1
    Tn = model["n_op_types"]
    # Large bf16 batches run on the forward kernels that keep relu(z1) and the ReLU mask bits of z1
    # and y for the backward pass, and on the backward kernels that start from the bits.
    kept = (backward and bf16 and args.round_kind == "mlp" and kern["resident"]["launches_per_step"] == 0
            and min(N, E) >= int(os.environ.get("XRL_PERSISTENT_MIN_ROWS", 8192)))
    zk = 1 if kept else 0
    # Algorithmic work per launch of each kernel (multiply-add = 2 flop; b = bytes per stored
    # activation): flops of the products the kernel is there for, and the bytes of its inputs read
    # once and its outputs written once (rows gathered several times count once). A kernel whose
    # flops / bytes lies below the ridge of the two peaks is rated against HBM, else against the
    # matrix cores.
    NH, EH = N * H * b, E * H * b
    idx_e = 4 * (2 * E + n_tiles)
    # the kept forward's mask bits of one MLP's z1 or y: 16 bits per lane, 32-feature block and wave tile
    mask_e, mask_n = n_tiles * (H // 32) * 128, ((N + 31) // 32) * (H // 32) * 128
    work = {
        "embed": dict(kernel="node-update layer: sum of incoming edge attributes + embed MLP",
                      flops=2.0 * N * H * (De + Dd + H),
                      bytes=E * De * 4 + N * (4 + 4 * Dd) + 4 * (N + 1) + NH * (1 + zk) + zk * 2 * mask_n),
        "edge": dict(kernel="edge MLP + per-receiver sum (one launch per round)",
                     flops=2.0 * E * H * (3 * H + De),
                     bytes=NH + E * De * 4 + idx_e + n_recv * H * b + zk * (EH + 2 * mask_e)),
        "node": dict(kernel="node MLP (one launch per round)", flops=2.0 * N * H * 3 * H,
                     bytes=(2 + zk) * NH + n_recv * H * b + 4 * N + zk * 2 * mask_n),   # received sums: nodes with in-edges only
        "pool": dict(kernel="per-graph readout sum (fused with the readout MLP)", flops=0.0,
                     bytes=NH + 4 * (G + 1) + G * H * 4),
        "grad_gather": dict(kernel="per-node sum of the per-edge gradients (receiver and sender side)", flops=0.0,
                            bytes=(EH + n_recv * H * b + mask_n if kept else 2 * EH) + 2 * NH + 4 * (2 * N + E)),
    }
    if kept:
        work.update({
            "bwd_edge": dict(kernel="backward through the edge MLP from the kept forward (one launch per round)",
                             flops=2.0 * E * H * 3 * H,
                             bytes=n_recv * H * b + 2 * mask_e + 4 * (E + n_tiles) + 3 * EH + n_recv * H * b),
            "bwd_node": dict(kernel="backward through the node MLP from the kept forward (one launch per round)",
                             # dz2 arrives masked from the gradient gather and is read (NH) instead of stored; the
                             # topmost round reads the per-graph table and stores dz2 itself (NH either way);
                             # dz1, dh, and the dagg rows of the nodes with in-edges are written
                             flops=2.0 * N * H * 3 * H,
                             bytes=3 * NH + n_recv * H * b + mask_n * (1 + 1 / max(R, 1)) + 4 * N),
            "bwd_embed": dict(kernel="backward through the embed MLP from the kept forward", flops=2.0 * N * H * H,
                              bytes=2 * NH + mask_n),
            "wgrad_edge": dict(kernel="weight gradients of one edge MLP, both layers",
                               flops=2.0 * E * H * (3 * H + De + 2), bytes=NH + 4 * EH + E * De * 4 + 8 * E),
            "wgrad_node": dict(kernel="weight gradients of one node MLP, both layers",
                               flops=2.0 * N * H * (3 * H + 2), bytes=4 * NH + n_recv * H * b + 4 * N),
            "wgrad_embed": dict(kernel="weight gradients of the embed MLP, both layers",
                                flops=2.0 * N * H * (De + Tn + Dd + H + 2), bytes=3 * NH + E * De * 4 + N * (8 + 4 * Dd)),
        })
    else:
        # small batches and fp32: the backward kernels recompute the first layer (and, for the edge
        # kind, the second) of the forward on the matrix cores; that recomputation is counted
        work.update({
            "bwd_edge": dict(kernel="backward through the edge MLP (one launch per round)", flops=2.0 * E * H * (6 * H + De),
                             bytes=None),
            "bwd_node": dict(kernel="backward through the node MLP (one launch per round)", flops=2.0 * N * H * 5 * H, bytes=None),
            "bwd_embed": dict(kernel="backward through the embed MLP", flops=2.0 * N * H * (De + Dd + 2 * H), bytes=None),
            "wgrad_edge": dict(kernel="weight gradients of one edge MLP, both layers", flops=2.0 * E * H * (3 * H + De + 2), bytes=None),
            "wgrad_node": dict(kernel="weight gradients of one node MLP, both layers", flops=2.0 * N * H * (3 * H + 2), bytes=None),
            "wgrad_embed": dict(kernel="weight gradients of the embed MLP, both layers",
                                flops=2.0 * N * H * (De + Tn + Dd + H + 2), bytes=None),
        })
    ridge = peak * 1e12 / (PEAK_HBM_GBS * 1e9)           # flop per byte at which the two peaks meet
    report = {}
    for k, wk in work.items():
        if k not in kern or kern[k]["launches_per_step"] == 0 or kern[k]["avg_us"] <= 0:
            continue
        sec = kern[k]["avg_us"] * 1e-6
        e = dict(kernel=wk["kernel"], avg_launch_us=kern[k]["avg_us"], launches_per_step=kern[k]["launches_per_step"],
                 share_of_step=kern[k]["avg_us"] * kern[k]["launches_per_step"] * 1e-3 / ms)
        hbm = wk["bytes"] is not None and (wk["flops"] == 0 or wk["flops"] / wk["bytes"] < ridge)
        if hbm:
            e.update(bound="hbm", achieved=wk["bytes"] / sec / 1e9, peak=PEAK_HBM_GBS, unit="GB/s",
                     algorithmic_bytes_per_launch=wk["bytes"])
            if wk["flops"]:
                e.update(flops_per_launch=wk["flops"], mfma_frac=wk["flops"] / sec / 1e12 / peak)
        else:
            e.update(bound="mfma", achieved=wk["flops"] / sec / 1e12, peak=peak, unit="TFLOP/s", flops_per_launch=wk["flops"])
            if wk["bytes"] is not None:
                e.update(algorithmic_bytes_per_launch=wk["bytes"], hbm_frac=wk["bytes"] / sec / 1e9 / PEAK_HBM_GBS)
        e["frac"] = e["achieved"] / e["peak"]
        e["traffic"] = measured_traffic(args.config, model["precision"], k)
        report[k] = e

    res = dict(
        metric="candidate graphs encoded/sec on 1 MI355X", value=G / (ms * 1e-3), unit="graphs/s",
        n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=ms, ms_per_step_mean=ms_mean,
        higher_is_better=True, scaling="weak", vs_baseline=None, dtype=model["precision"], data="synthetic",
        config=dict(workload=f"config {args.config} ({synth.CONFIGS[args.config]['name']}): {S} state(s), "
                             f"{G} graphs, {N} nodes, {E} edges, hidden {H}, {R} rounds, forward "
                             f"(encode + policy/value heads)" + (" + backward (heads, encoder)" if backward else ""),
                    states=S, graphs=G, nodes=N, edges=E, hidden=H, rounds=R),
        edges_per_s=E * R / (ms * 1e-3),
        pack_upload_ms=t_pack * 1e3,              # host packing + H2D copies, outside the timed region
        kernels_us=kern,
    )
    if report:
        # the roofline entry rates the kernel that takes the largest share of the step
        top = max(report, key=lambda k: report[k]["share_of_step"])
        res["roofline"] = report[top]
        res["kernels"] = {k: v for k, v in report.items() if k != top}
    if kern["resident"]["launches_per_step"] > 0:
        # small batch: the encoder ran as one launch (a block per graph), rated as a whole
        enc_flops = 2.0 * N * H * (De + Tn + Dd + H) + R * (work["edge"]["flops"] + 2.0 * N * H * 3 * H)
        enc_s = kern["resident"]["avg_us"] * 1e-6
        enc_bytes = (R + 1) * N * H * b + R * n_recv * H * b + E * De * 4 + 4 * (3 * E + 3 * N) + G * H * 4
        res["roofline"] = dict(bound="mfma", kernel="one-launch encoder (node-update layer, all rounds, readout)",
                               achieved=enc_flops / enc_s / 1e12, peak=peak, unit="TFLOP/s",
                               frac=enc_flops / enc_s / 1e12 / peak, traffic=None, flops_per_launch=enc_flops,
                               avg_launch_us=kern["resident"]["avg_us"], algorithmic_bytes_per_launch=enc_bytes,
                               hbm_frac=enc_bytes / enc_s / 1e9 / PEAK_HBM_GBS)
    if args.round_kind == "gat":
        # attention rounds: the dense part z = h W on the matrix cores, then a gather-bound pass
        # (per edge one z row read, per node its own row read and one row written, scores, indices)
        agg_bytes = (E + 2 * N) * H * b + 4 * (2 * N + 2 * E)
        agg_s, lin_s = kern["gat_aggregate"]["avg_us"] * 1e-6, kern["gat_linear"]["avg_us"] * 1e-6
        res["config"]["workload"] += ", graph-attention rounds"
        res["roofline"] = dict(bound="hbm", kernel="attention-weighted sum over in-edges (one launch per round)",
                               achieved=agg_bytes / agg_s / 1e9, peak=PEAK_HBM_GBS, unit="GB/s",
                               frac=agg_bytes / agg_s / 1e9 / PEAK_HBM_GBS, traffic=None,
                               algorithmic_bytes_per_launch=agg_bytes, avg_launch_us=kern["gat_aggregate"]["avg_us"])
        res["mfma_kernel"] = dict(kernel="z = h W (one launch per round)", flops_per_launch=2.0 * N * H * H,
                                  achieved=2.0 * N * H * H / lin_s / 1e12, peak=peak, unit="TFLOP/s",
                                  frac=2.0 * N * H * H / lin_s / 1e12 / peak, avg_launch_us=kern["gat_linear"]["avg_us"])
    if not args.no_segment_sum and E > 0:
        # the receiver-side sum on its own: an [E, H] fp32 message tensor in receiver order summed
        # into [N, H] (xrl_segment_sum), 5 launches after one warm-up
        vals = torch.empty((E, H), dtype=torch.float32, device="cuda").normal_()
        ptr = torch.from_numpy(hv["in_ptr"]).cuda()
        out = torch.empty((N, H), dtype=torch.float32, device="cuda")
        enc.segment_sum(vals, ptr, out=out)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            enc.segment_sum(vals, ptr, out=out)
        e1.record()
        torch.cuda.synchronize()
        seg_s = e0.elapsed_time(e1) * 1e-3 / 5
        seg_bytes = E * H * 4 + 4 * (N + 1) + N * H * 4
        res["segment_sum"] = dict(kernel="standalone receiver-side sum of an [E, H] fp32 tensor (segment-sum + carry fix-up)",
                                  bound="hbm", algorithmic_bytes_per_launch=seg_bytes, avg_launch_us=seg_s * 1e6,
                                  achieved=seg_bytes / seg_s / 1e9, peak=PEAK_HBM_GBS, unit="GB/s",
                                  frac=seg_bytes / seg_s / 1e9 / PEAK_HBM_GBS)
        del vals, out
    if args.edit_pack:
        # host packing + H2D of one rewrite step's state, both ways (best of 40 after one warm-up)
        erng = np.random.Generator(np.random.PCG64(synth.BASE_SEED + 11))
        base = synth.shuffle_edges(erng, synth.transformer_dag(erng, 12))
        edit_state, full_state = synth.make_edit_states(erng, [base], 128)
        em = dict(model, hidden=128)
        eenc = xrl.Encoder(em, synth.init_weights(erng, xrl.weight_layout(em)))

        def best(fn):
            ts = []
            for _ in range(41):
                t0 = time.perf_counter()
                bt = fn()
                torch.cuda.synchronize()
                ts.append(time.perf_counter() - t0)
                bt.free()
            return min(ts[1:]) * 1e3
        res["edit_pack"] = dict(workload=f"1 state, 128 candidates of a {base.n_nodes}-node / {base.n_edges}-edge graph",
                                whole_graphs_ms=best(lambda: eenc.pack(full_state)),
                                edits_ms=best(lambda: eenc.pack_edits(edit_state)),
                                note="host packing + upload; the marshalling of the numpy arrays is included on both sides")
        eenc.close()
    if args.peaks:
        tf, gb = enc.measure_peaks()
        res["measured_peaks"] = dict(mfma_bf16_tflops=tf, copy_gbs=gb,
                                     note="register-resident 32x32x16 bf16 MFMA loop; 1 GiB device copy, read + write")
    if not args.no_cpu_baseline:
        if backward and args.round_kind == "mlp":
            res["cpu_baseline"] = oracle_baseline_update(model, state, w, up_host, min(args.cpu_baseline_states, S))
        else:
            res["cpu_baseline"] = oracle_baseline_forward(model, state, w, args.cpu_baseline_seconds)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
