"""GPU parity of the backward path (heads, then encoder) against the oracle's hand-written
reverse mode (itself pinned by finite differences in test_oracle_pins.py), through the C ABI.

fp32 path, end to end (heads + encoder, loss = sum c.logp + d.value + f.entropy), per weight
tensor and element-wise (grad_checks.check_fp32):
    |g - ref| <= 1e-5 |ref| + 1e-5 scale + 2e-6 B + A
  B = the sum of the absolute terms the entry is made of (returned by the oracle), A = the
  per-mask allowance: non-zero only where a pre-activation of the oracle lies within 1e-5 of its
  layer's scale of zero, in which case the GPU's fp32 forward may take the other ReLU mask; the
  oracle's reverse mode is re-run with that one mask inverted and the change is allowed.
bf16 path: the backward pass multiplies by ReLU masks taken from the bf16 forward. With random
  weights about 0.4 % of the pre-activations lie within the forward's rounding error of zero and
  get the opposite mask from the float64 oracle, each flipped term entering the gradient in full
  (about sqrt(0.004) = 6 % relative L2 error per tensor whatever the backward arithmetic does), so
  the element-wise criterion is asserted on mask-stable cases: weights under which every
  pre-activation of the oracle is at least 0.25 away from zero (all units on; or units on/off per
  feature and, in the node-update layer, per operator type), where both sides differentiate the
  same piecewise-linear function (grad_checks.check_bf16_elementwise: the stated tolerance as it
  is where no sum cancels, plus 4e-5 of the chain's sum of absolute terms where sums cancel), at
  H = 64 / 128 / 256, with hubs and empty graphs, and on
  sampled graphs of the full update minibatch. The same cases run in fp32 at the fp32 criterion
  with no allowance at all. On random weights the bf16 runs assert, per tensor, relative L2 error
  <= 0.15 and cosine >= 0.98 (the statistical complement), plus the exact parts (masked rows zero,
  heads in fp32, accumulation into the buffer, run-to-run determinism).
"""
import numpy as np
import pytest

import synth
from oracle import xrl_oracle as O
import grad_checks as GC
from test_gpu_forward import oracle_model, weights_for, hub_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xrl():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2304_14698_amd as x
    x.load_library()
    return x


def tensors(model):
    for name, sl, _ in GC.tensors(oracle_model(model)):
        yield name, sl


def check_grads(got, ref, bound, model, only=None, allowance=None, kappa=2e-6):
    """fp32 criterion (see the module docstring)."""
    GC.check_fp32(got, ref, bound, oracle_model(model), allowance=allowance, only=only, kappa=kappa)


def check_grads_bf16(got, ref, model, only, max_rel=0.15, min_cos=0.98):
    bad = []
    gnorm = np.linalg.norm(ref)
    for name, sl in tensors(model):
        if not name.startswith(only):
            continue
        g, r = got[sl].astype(np.float64), ref[sl]
        if np.linalg.norm(r) < 1e-3 * gnorm:
            continue
        rel = np.linalg.norm(g - r) / np.linalg.norm(r)
        if rel > max_rel or cosine(g, r) < min_cos:
            bad.append(f"{name}: relative L2 error {rel:.3f}, cosine {cosine(g, r):.4f}")
    assert not bad, "\n".join(bad)


def cosine(a, b):
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b) + 1e-300))


def run_backward_case(xrl, model, state, w, seed=3, bf16_rel=0.15, bf16_cos=0.98):
    """Heads + encoder backward of loss = sum c.logp + d.value + f.entropy against the oracle's own
    chain (its forward, its heads' reverse mode, its encoder's), then the encoder alone on a given
    random upstream embedding gradient (the same array on both sides).

    Chain, fp32: the upstream embedding gradient comes from a softmax whose probabilities carry a
    relative error of 1e-5 L (L = the largest |logit|; the forward's tolerance on logp), and every
    gradient is linear in it; the logits' own error is relative to the embeddings' scale rather
    than to L where the logits are small (measured: 2.8e-5 B on a case with L = 0.12), so the B
    term's factor is 4e-5 + 1e-5 L.
    Encoder alone, fp32: the plain criterion, factor 2e-6."""
    import torch
    prec = model["precision"]
    om = oracle_model(model)
    G, S = len(state["slot_mask"]), state["n_states"]
    rng = np.random.Generator(np.random.PCG64(seed))
    dlogp, dvalue, dentropy = synth.upstream_grads(rng, G, S)
    enc = xrl.Encoder(model, w)
    batch = enc.pack(state)
    emb = enc.encode(batch, save_for_backward=True)
    dw = torch.zeros(enc.n_weights, dtype=torch.float32, device="cuda")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    demb = enc.policy_value_backward(batch, emb, t(dlogp), t(dvalue), t(dentropy), dw)
    torch.cuda.synchronize()
    dw_heads = dw.cpu().numpy().copy()
    enc.encode_backward(batch, demb, dw)
    torch.cuda.synchronize()
    dw_all = dw.cpu().numpy().copy()

    head_names = ("policy", "value")
    n_head = sum(int(np.prod(s)) for n, s in O.weight_layout(om) if n.startswith(head_names))
    assert np.all(dw_heads[:len(dw_heads) - n_head] == 0), "the heads' backward wrote encoder gradients"
    mask = state["slot_mask"] == 1
    d = demb.cpu().numpy()
    assert np.all(d[~mask] == 0.0), "masked slots must get exactly zero gradient"
    ba = O.zero_grads(om)
    _, ref_all, ref_demb = O.loss_and_grad(om, w, state, dlogp, dvalue, dentropy, bound=ba)
    L = float(np.abs(O.policy_value(om, w, O.encode(om, w, state), state)["logit"]).max())
    names = tuple(n for n, _ in O.weight_layout(om) if not n.startswith(head_names))
    gat = model.get("round_kind", "mlp") == "gat"
    # (attention rounds: the softmax gradient sums to zero over a receiver's edges, a cancellation
    # inside the factors that B does not see: absolute term 5e-5 of the tensor's scale)
    atol = 5e-5 if gat else 1e-5
    if prec == "fp32":
        np.testing.assert_allclose(d, ref_demb, rtol=1e-4, atol=1e-5 * max(1.0, L) * np.abs(ref_demb).max())
        A, n_near = GC.flip_allowance(om, w, state, ref_demb)
        Ah, n_heads = GC.heads_flip_allowance(om, w, O.encode(om, w, state), state, dlogp, dvalue, dentropy)
        A = A + Ah
        # the heads' first layers multiply the embeddings, which the forward holds to 1e-5 of their
        # scale and no better (a feature that is nearly off has an error far above 1e-5 of its own
        # value): dW0[k, f] may be off by that times sum_g |dz[g, f]|, which is the bound of db0[f]
        emb_scale = float(np.abs(O.encode(om, w, state)).max())
        bflat = O.flatten(om, ba)
        tens = {name: (sl, shape) for name, sl, shape in GC.tensors(om)}
        for head in head_names:
            slw, shape = tens[f"{head}.W0"]
            slb, _ = tens[f"{head}.b0"]
            A[slw] += (1e-5 * emb_scale * np.broadcast_to(bflat[slb], shape)).ravel()
        print(f"undecided ReLU masks (|z| <= 1e-5 scale) in the oracle: {n_near} in the encoder, {n_heads} in the heads; "
              f"largest |logit| {L:.3g}")
        GC.check_fp32(dw_all, ref_all, O.flatten(om, ba), om, allowance=A, kappa=4e-5 + 1e-5 * L, atol=atol)
    else:
        assert cosine(dw_all.astype(np.float64), ref_all) >= 0.9
    # the encoder alone: a given upstream embedding gradient, the same on both sides
    rdemb = rng.standard_normal((G, model["hidden"])).astype(np.float32)
    dwr = torch.zeros_like(dw)
    enc.encode_backward(batch, t(rdemb), dwr)
    torch.cuda.synchronize()
    br = O.zero_grads(om)
    ref_r = O.encode_backward(om, w, state, rdemb.astype(np.float64), bound=br)
    if prec == "fp32":
        A, n_near = GC.flip_allowance(om, w, state, rdemb.astype(np.float64))
        GC.check_fp32(dwr.cpu().numpy(), ref_r, O.flatten(om, br), om, allowance=A, only=names, atol=atol)
    else:
        check_grads_bf16(dwr.cpu().numpy(), ref_r, model, names, bf16_rel, bf16_cos)

    # the gradient buffer is accumulated into, and the result is run-to-run identical
    emb2 = enc.encode(batch, save_for_backward=True)
    dw2 = torch.zeros_like(dw)
    demb2 = enc.policy_value_backward(batch, emb2, t(dlogp), t(dvalue), t(dentropy), dw2)
    enc.encode_backward(batch, demb2, dw2)
    torch.cuda.synchronize()
    assert torch.equal(dw2, dw), "two backward runs differ"
    enc.encode_backward(batch, demb2, dw2)
    torch.cuda.synchronize()
    enc_part = dw2.cpu().numpy() - dw_all
    np.testing.assert_allclose(enc_part, dw_all - dw_heads, rtol=1e-5, atol=1e-6 * np.abs(dw_all).max())
    batch.free()
    enc.close()


def test_backward_config1_fp32(xrl):
    model, state = synth.make_config(1)
    run_backward_case(xrl, model, state, weights_for(model))


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_backward_transformer_small(xrl, precision):
    model, state = synth.make_config(2, n_cand=10)
    model["precision"] = precision
    run_backward_case(xrl, model, state, weights_for(model))


@pytest.mark.parametrize("hidden,precision,readout", [(64, "bf16", "sum"), (256, "fp32", "mean"),
                                                      (256, "bf16", "sum")])
def test_backward_other_widths(xrl, hidden, precision, readout):
    model, state = synth.make_config(4, n_cand=3)
    model.update(hidden=hidden, precision=precision, rounds=2, readout=readout)
    run_backward_case(xrl, model, state, weights_for(model))


@pytest.mark.parametrize("cfg,hidden,precision", [(1, 64, "fp32"), (2, 128, "bf16"), (4, 256, "bf16"),
                                                  (4, 128, "fp32")])
def test_backward_graph_attention_rounds(xrl, cfg, hidden, precision):
    """The graph-attention reading of the rounds: softmax and score gradients per receiver, dz per
    sender, the two dense products. fp32: the elementwise criterion of the MLP rounds. bf16: the
    per-tensor criterion with wider thresholds -- an attention round has no bias and puts its
    ReLU directly on a convex combination of z rows, so more pre-activations lie within the bf16
    forward's rounding error of zero than in an MLP round; the gradients of the readout MLP,
    computed in fp32 from that forward, are already 15-16 % (relative L2) away from the float64
    oracle's, and the attention weights' gradients show the same 16-17 %."""
    model, state = synth.make_config(cfg, n_cand=12 if cfg != 1 else None)
    model.update(hidden=hidden, precision=precision, rounds=2, round_kind="gat")
    run_backward_case(xrl, model, state, weights_for(model), bf16_rel=0.3, bf16_cos=0.95)


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_backward_paper_feature_dimensions(xrl, precision):
    """Backward with the state description the paper prints: 40 operator types, no other node
    attributes, 4 edge attributes (shape over 4096), zero global attribute."""
    model, state = synth.make_config(2, n_cand=5)
    model.update(hidden=128, precision=precision, rounds=2, n_op_types=40, n_node_dense=0, d_edge=4)
    rng = np.random.Generator(np.random.PCG64(31))
    E, N = len(state["edge_src"]), len(state["node_op"])
    extents = np.array([1, 3, 12, 64, 128, 197, 256, 768, 1000, 3072])
    shapes = [list(rng.choice(extents, size=int(rng.integers(1, 5)))) for _ in range(E)]
    state = dict(state, node_op=rng.integers(0, 40, N).astype(np.int32), node_dense=np.zeros((N, 0), np.float32),
                 edge_feat=xrl.edge_features_from_shapes(shapes),
                 graph_global=np.zeros((len(state["slot_mask"]), model["d_global"]), np.float32))
    run_backward_case(xrl, model, state, weights_for(model))


@pytest.mark.parametrize("round_kind,cfg,hidden,precision", [("gat", 1, 64, "fp32"), ("gat", 2, 128, "bf16"),
                                                             ("mlp", 1, 64, "fp32"), ("mlp", 2, 128, "bf16"),
                                                             ("mlp", 4, 256, "bf16")])
def test_backward_single_learned_matrix_per_layer(xrl, round_kind, cfg, hidden, precision):
    """mlp_layers = 1 (Section 3.4's layers with their single learned matrix; with graph-attention
    rounds the network as printed): gradients of every tensor of the one-layer layout against the
    oracle's reverse mode, criteria of the two-layer cases. The library differentiates its
    two-layer kernels with an identity second layer and drops that layer's gradient."""
    model, state = synth.make_config(cfg, n_cand=12 if cfg != 1 else None)
    model.update(hidden=hidden, precision=precision, rounds=2, round_kind=round_kind, mlp_layers=1)
    gat = round_kind == "gat"
    run_backward_case(xrl, model, state, weights_for(model), bf16_rel=0.3 if gat else 0.15, bf16_cos=0.95 if gat else 0.98)


@pytest.mark.parametrize("hidden", [128, 256])
def test_backward_wide_weight_gradient_tiles(xrl, hidden, monkeypatch):
    """The 256-column tiles of the weight-gradient kernel (used from 2^20 rows on) forced onto a
    small batch, where row slices are short and ragged."""
    monkeypatch.setenv("XRL_WGRAD_WIDE_MIN_ROWS", "0")
    model, state = synth.make_config(4, n_cand=3)
    model.update(hidden=hidden, precision="bf16", rounds=2)
    run_backward_case(xrl, model, state, weights_for(model))


def test_backward_ppo_minibatch_subset_bf16(xrl):
    """Two states of the PPO-minibatch configuration with a reduced candidate count."""
    model, state = synth.make_config(5, n_states=2, n_cand=12)
    model["rounds"] = 3
    run_backward_case(xrl, model, state, weights_for(model))


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_backward_hubs_and_empty_graphs(xrl, precision):
    rng = np.random.Generator(np.random.PCG64(5))
    model, _ = synth.make_config(1)
    model.update(precision=precision, hidden=64, rounds=2)
    state = hub_state(rng, model, 150)
    # five small graphs (about 250 nodes): with so few rows a single flipped ReLU mask is a
    # visible share of a gradient entry, so the bf16 thresholds are loose here; the exact
    # handling of hubs, empty graphs and carries is asserted by the fp32 variant
    run_backward_case(xrl, model, state, weights_for(model) * 0.5, bf16_rel=0.8, bf16_cos=0.75)


def test_backward_needs_saved_forward(xrl):
    import torch
    model, state = synth.make_config(1)
    enc = xrl.Encoder(model, weights_for(model))
    batch = enc.pack(state)
    emb = enc.encode(batch, save_for_backward=False)
    dw = torch.zeros(enc.n_weights, device="cuda")
    with pytest.raises(xrl.XrlError) as ei:
        enc.encode_backward(batch, torch.zeros_like(emb), dw)
    assert ei.value.code == xrl.ERR["STATE"]
    torch.cuda.synchronize()


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_backward_full_size_sampled_graphs(xrl, cfg):
    """Configurations 3-5 at full size, in the launch configuration the benchmark times. The
    upstream embedding gradient is non-zero on a few sampled graphs only; graphs are independent,
    so the weight gradient must equal the oracle's over those graphs alone (bf16 criterion of
    this module), while every other row of the batch goes through the same launches with zero
    gradients -- a contribution picked up from a wrong row would show. Also run-to-run identical."""
    import torch
    model, state = synth.make_config(cfg)
    assert model["precision"] == "bf16"
    w = weights_for(model)
    om = oracle_model(model)
    enc = xrl.Encoder(model, w)
    batch = enc.pack(state)
    enc.encode(batch, save_for_backward=True)
    G = batch.G
    rng = np.random.Generator(np.random.PCG64(23 + cfg))
    sample = sorted(set([0, G - 1] + rng.integers(0, G, 4).tolist()))
    demb = np.zeros((G, model["hidden"]), np.float32)
    demb[sample] = rng.standard_normal((len(sample), model["hidden"])).astype(np.float32)
    d_demb = torch.from_numpy(demb).cuda()
    dw = torch.zeros(enc.n_weights, dtype=torch.float32, device="cuda")
    enc.encode_backward(batch, d_demb, dw)
    torch.cuda.synchronize()
    got = dw.cpu().numpy()
    assert np.isfinite(got).all()
    ref = O.encode_backward(om, w, state, demb[sample].astype(np.float64), graphs=sample)   # (demb indexed by position)
    names = tuple(n for n, _ in O.weight_layout(om) if not n.startswith(("policy", "value")))
    check_grads_bf16(got, ref, model, names)
    dw2 = torch.zeros_like(dw)
    enc.encode_backward(batch, d_demb, dw2)
    torch.cuda.synchronize()
    assert torch.equal(dw, dw2), "two backward runs differ"
    batch.free()
    enc.close()


def run_stable_case(xrl, model, state, kind, seed=7, graphs=None, max_indeg=8, max_nodes=1500):
    """xrl_encode_backward on a mask-stable case (see the module docstring) against the oracle,
    element-wise. `graphs`: the upstream gradient is non-zero on these graphs only and the oracle
    runs on them alone."""
    import torch
    om = oracle_model(model)
    if kind == "all_on":
        state = dict(state, edge_feat=np.abs(state["edge_feat"]), graph_global=np.abs(state["graph_global"]))
    w = GC.stable_weights(om, kind, seed, max_indeg=max_indeg, max_nodes=max_nodes)
    margin, on = GC.min_margin(om, w, state, graphs=graphs)
    assert margin >= (0.25 if kind == "fixed" else 0.04), f"smallest |pre-activation| {margin}"
    assert on == 1.0 if kind == "all_on" else 0.3 < on < 0.7, on
    G, H = len(state["slot_mask"]), model["hidden"]
    rng = np.random.Generator(np.random.PCG64(seed + 1))
    sel = list(range(G)) if graphs is None else list(graphs)
    demb = np.zeros((G, H), np.float32)
    demb[sel] = rng.standard_normal((len(sel), H)).astype(np.float32)
    if kind == "all_on":
        demb = np.abs(demb)                      # no term of any sum cancels
    enc = xrl.Encoder(model, w)
    batch = enc.pack(state)
    enc.encode(batch, save_for_backward=True)
    dw = torch.zeros(enc.n_weights, dtype=torch.float32, device="cuda")
    enc.encode_backward(batch, torch.from_numpy(demb).cuda(), dw)
    torch.cuda.synchronize()
    got = dw.cpu().numpy()
    bd = O.zero_grads(om)
    ref = O.encode_backward(om, w, state, demb[sel].astype(np.float64), graphs=sel, bound=bd)
    names = tuple(n for n, _ in O.weight_layout(om) if not n.startswith(("policy", "value")))
    if model["precision"] == "fp32":
        GC.check_fp32(got, ref, O.flatten(om, bd), om, only=names)
    elif kind == "all_on":
        GC.check_bf16_elementwise(got, ref, om)
    else:
        C = GC.abs_chain_bound(om, w, state, demb[sel].astype(np.float64), graphs=sel)
        worst = GC.check_bf16_elementwise(got, ref, om, chain_bound=C)
        print(f"largest (error - 2e-2 |ref| - 1e-3 scale) / C: {worst:.3e}")
    batch.free()
    enc.close()


@pytest.mark.parametrize("kind", ["all_on", "fixed"])
@pytest.mark.parametrize("hidden,precision", [(64, "bf16"), (128, "bf16"), (256, "bf16"), (64, "fp32"), (128, "fp32")])
def test_backward_elementwise_on_mask_stable_cases(xrl, hidden, precision, kind):
    model, state = synth.make_config(4, n_cand=3)
    model.update(hidden=hidden, precision=precision, rounds=3)
    run_stable_case(xrl, model, state, kind)


@pytest.mark.parametrize("kind", ["all_on", "fixed"])
@pytest.mark.parametrize("hidden,readout", [(64, "sum"), (256, "mean")])
def test_backward_elementwise_hubs_bf16(xrl, hidden, readout, kind):
    """A receiver of in-degree 150 (split over several edge tiles), zero-edge, single-node and
    empty graphs, bf16, element-wise."""
    rng = np.random.Generator(np.random.PCG64(5))
    model, _ = synth.make_config(1)
    model.update(precision="bf16", hidden=hidden, rounds=2, readout=readout)
    run_stable_case(xrl, model, hub_state(rng, model, 150), kind, max_indeg=160, max_nodes=200)


@pytest.mark.parametrize("hidden,precision,kind", [(128, "bf16", "fixed"), (128, "fp32", "fixed"), (64, "bf16", "fixed"),
                                                   (256, "bf16", "fixed"), (256, "bf16", "all_on"), (128, "bf16", "all_on")])
def test_backward_elementwise_persistent_kernels(xrl, hidden, precision, kind, monkeypatch):
    """The kernels of large batches forced onto a transformer-shaped state of 12 candidates: the
    persistent forward kernels, which in bf16 keep z1 and the ReLU masks, the backward from what
    they kept, and the wide weight-gradient tiles; element-wise on mask-stable cases."""
    monkeypatch.setenv("XRL_PERSISTENT_MIN_ROWS", "0")
    monkeypatch.setenv("XRL_WGRAD_WIDE_MIN_ROWS", "0")
    model, state = synth.make_config(2, n_cand=12)
    model.update(precision=precision, hidden=hidden, rounds=5 if hidden == 128 else 3)
    run_stable_case(xrl, model, state, kind)


@pytest.mark.parametrize("hidden", [64, 256])
def test_backward_kept_forward_hubs_and_random_weights(xrl, hidden, monkeypatch):
    """The backward from what the forward kept (bf16, large-batch kernels forced): a receiver of
    in-degree 150 split over several edge tiles, zero-edge, single-node and empty graphs,
    element-wise on a mask-stable case; then random weights on an Inception-shaped state at the
    per-tensor criterion, including the chain through the heads and run-to-run identity."""
    monkeypatch.setenv("XRL_PERSISTENT_MIN_ROWS", "0")
    rng = np.random.Generator(np.random.PCG64(5))
    model, _ = synth.make_config(1)
    model.update(precision="bf16", hidden=hidden, rounds=2)
    run_stable_case(xrl, model, hub_state(rng, model, 150), "fixed", max_indeg=160, max_nodes=200)
    model, state = synth.make_config(4, n_cand=3)
    model.update(hidden=hidden, precision="bf16", rounds=2)
    run_backward_case(xrl, model, state, weights_for(model))


def test_backward_elementwise_update_minibatch_full_size(xrl):
    """The update minibatch (configuration 5) at full size, bf16, element-wise: mask-stable
    weights, upstream gradient on sampled graphs, the oracle on those graphs alone."""
    model, state = synth.make_config(5)
    G = len(state["slot_mask"])
    rng = np.random.Generator(np.random.PCG64(29))
    sample = sorted(set([0, G - 1] + rng.integers(0, G, 3).tolist()))
    run_stable_case(xrl, model, state, "fixed", graphs=sample)
