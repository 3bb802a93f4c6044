"""Pins of the float64 oracle against things other than itself: a hand-worked example,
dense-matrix brute force, closed forms, invariances, adjoint identities, finite differences."""
import os
import numpy as np
import pytest

from oracle import xrl_oracle as O
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ small random inputs
def tiny_model(**kw):
    m = O.default_model(n_op_types=5, n_node_dense=2, d_edge=3, d_global=1, hidden=8, rounds=2,
                        mlp_layers=2, head_hidden=(12, 6))
    m.update(kw)
    return m


def rand_graph(rng, model, n, e, allow_multi=True):
    op = rng.integers(0, model["n_op_types"], size=n).astype(np.int32)
    dense = rng.integers(0, 13, size=(n, model["n_node_dense"])).astype(np.float64)
    src = rng.integers(0, max(n, 1), size=e).astype(np.int32)
    dst = rng.integers(0, max(n, 1), size=e).astype(np.int32)
    xe = rng.standard_normal((e, model["d_edge"]))
    return op, dense, src, dst, xe


def state_of(model, graphs, counts, mask=None):
    """graphs: list of (op, dense, src, dst, xe); counts: graphs per state."""
    gnp = np.concatenate([[0], np.cumsum([g[0].shape[0] for g in graphs])]).astype(np.int32)
    gep = np.concatenate([[0], np.cumsum([g[2].shape[0] for g in graphs])]).astype(np.int32)
    sgp = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    G = len(graphs)
    return dict(n_states=len(counts), state_graph_ptr=sgp, graph_node_ptr=gnp, graph_edge_ptr=gep,
                node_op=np.concatenate([g[0] for g in graphs]).astype(np.int32),
                node_dense=np.concatenate([g[1].reshape(g[0].shape[0], model["n_node_dense"]) for g in graphs]),
                edge_src=np.concatenate([g[2] for g in graphs]).astype(np.int32),
                edge_dst=np.concatenate([g[3] for g in graphs]).astype(np.int32),
                edge_feat=np.concatenate([g[4].reshape(g[2].shape[0], model["d_edge"]) for g in graphs]),
                graph_global=np.zeros((G, model["d_global"])),
                slot_mask=np.ones(G, dtype=np.uint8) if mask is None else np.asarray(mask, np.uint8))


def rand_weights(rng, model, bias=0.1):
    return synth.init_weights(rng, O.weight_layout(model), bias_range=bias).astype(np.float64)


def relu(x):
    return np.maximum(x, 0.0)


# ------------------------------------------------------------------ P2: hand-worked example
def read_golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        out[k] = np.array([float(t) for t in v])
    return out


def test_hand_example_matches_paper_layers():
    gold = read_golden("hand_example.txt")
    model = O.default_model(n_op_types=1, n_node_dense=0, d_edge=1, d_global=1, hidden=1,
                            rounds=1, mlp_layers=1, head_hidden=(4, 2))
    Wd = {n: np.ones(s) if len(s) == 2 else np.zeros(s) for n, s in O.weight_layout(model)}
    for head in ("policy", "value"):
        Wd[f"{head}.W0"][:] = 1 / 4
        Wd[f"{head}.W1"][:] = 1 / 2
    w = O.flatten(model, Wd)
    gA = (np.zeros(2, np.int32), np.zeros((2, 0)), np.array([0], np.int32), np.array([1], np.int32),
          np.array([[2.0]]))
    gB = (np.zeros(1, np.int32), np.zeros((1, 0)), np.zeros(0, np.int32), np.zeros(0, np.int32),
          np.zeros((0, 1)))
    st = state_of(model, [gA, gB], [2])
    emb, inter = O.encode(model, w, st, keep=True)
    a = inter[0]
    assert np.array_equal(a["a0"][:, 0], gold["a0"])
    assert np.array_equal(a["h"][0][:, 0], gold["h0"])
    assert np.array_equal(a["c_edge"][0][0][1][:, 0], gold["m"])
    assert np.array_equal(a["agg"][0][:, 0], gold["agg"])
    assert np.array_equal(a["h"][1][:, 0], gold["h1"])
    assert a["pool"][0] == gold["pool"][0]
    assert emb[0, 0] == gold["emb0"][0] and emb[1, 0] == gold["emb1"][0]
    pv = O.policy_value(model, w, emb, st)
    np.testing.assert_allclose(pv["logit"], gold["logit"], rtol=1e-14)
    np.testing.assert_allclose(pv["value"], gold["value"], rtol=1e-14)
    lp0 = -np.log1p(np.exp(-9.0))
    np.testing.assert_allclose(pv["logp"], [lp0, -9.0 + lp0], rtol=1e-13, atol=1e-14)
    assert pv["action"][0] == 0


# ------------------------------------------------------------------ P1: dense brute force
def dense_forward(model, W, op, dense, src, dst, xe, g):
    """The encoder written with dense incidence matrices only (no index arithmetic)."""
    n, e = op.shape[0], src.shape[0]
    B = np.zeros((n, e)); B[dst, np.arange(e)] = 1.0        # receiver incidence
    S = np.zeros((n, e)); S[src, np.arange(e)] = 1.0        # sender incidence
    X = np.concatenate([np.eye(model["n_op_types"])[op], dense], axis=1)
    def mlp(x, p):
        for i in range(model["mlp_layers"]):
            x = relu(x @ W[f"{p}.W{i}"] + W[f"{p}.b{i}"])
        return x
    Hm = mlp(np.concatenate([B @ xe, X], axis=1), "embed")
    for r in range(model["rounds"]):
        M = mlp(np.concatenate([S.T @ Hm, B.T @ Hm, xe], axis=1), f"edge{r}")
        Hm = mlp(np.concatenate([Hm, B @ M], axis=1), f"node{r}")
    pool = np.ones(n) @ Hm
    if model["readout"] == "mean":
        pool = pool / max(n, 1)
    return mlp(np.concatenate([pool, g])[None, :], "readout")[0]


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("readout", ["sum", "mean"])
def test_dense_incidence_twin(seed, readout):
    rng = np.random.default_rng(seed)
    model = tiny_model(readout=readout, rounds=3)
    w = rand_weights(rng, model)
    W = O.unflatten(model, w)
    for n, e in [(1, 0), (2, 1), (7, 15), (12, 30)]:
        op, dense, src, dst, xe = rand_graph(rng, model, n, e)
        g = rng.standard_normal(model["d_global"])
        got = O.encode_graph(model, W, op, dense, src, dst, xe, g)["emb"]
        ref = dense_forward(model, W, op, dense, src, dst, xe, g)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_round_reduces_to_adjacency_product():
    """Linear, bias-free, sender-only edge function: the received sum is A.H.W with
    A[i, j] = number of edges j -> i (non-negative values keep the ReLU inactive)."""
    rng = np.random.default_rng(3)
    model = tiny_model(mlp_layers=1, rounds=1)
    Wd = O.unflatten(model, rand_weights(rng, model))
    H, De = model["hidden"], model["d_edge"]
    We = np.zeros((2 * H + De, H)); We[:H] = rng.uniform(0, 1, size=(H, H))
    Wd["edge0.W0"], Wd["edge0.b0"] = We, np.zeros(H)
    op, dense, src, dst, xe = rand_graph(rng, model, 9, 25)
    out = O.encode_graph(model, Wd, op, dense, src, dst, xe, np.zeros(1))
    A = np.zeros((9, 9))
    for s, d in zip(src, dst):
        A[d, s] += 1.0
    np.testing.assert_allclose(out["agg"][0], A @ out["h"][0] @ We[:H], rtol=1e-12, atol=1e-12)
    assert (A.sum(axis=1) > 1).any()          # the case has real fan-in, incl. multi-edges


# ------------------------------------------------------------------ P12: printed first layer
def test_single_layer_paper_features():
    """One-hot of about 40 operators, 4 edge attributes, one W: h' = ReLU([sum e | onehot] W + b)."""
    rng = np.random.default_rng(4)
    model = O.default_model(n_op_types=40, n_node_dense=0, d_edge=4, hidden=6, rounds=0, mlp_layers=1,
                            head_hidden=(4, 2))
    w = rand_weights(rng, model)
    W = O.unflatten(model, w)
    op, dense, src, dst, xe = rand_graph(rng, model, 6, 9)
    xe = xe / 4096.0
    out = O.encode_graph(model, W, op, dense, src, dst, xe, np.zeros(1))
    for i in range(6):
        s = sum((xe[k] for k in range(9) if dst[k] == i), np.zeros(4))
        x = np.concatenate([s, np.eye(40)[op[i]]])
        np.testing.assert_allclose(out["h"][0][i], relu(x @ W["embed.W0"] + W["embed.b0"]), rtol=1e-12, atol=1e-15)


# ------------------------------------------------------------------ P3: zero-edge / zero-node
def test_zero_edge_and_zero_node_graphs():
    rng = np.random.default_rng(5)
    model = tiny_model()
    w = rand_weights(rng, model)
    W = O.unflatten(model, w)
    op, dense, _, _, _ = rand_graph(rng, model, 5, 0)
    none = np.zeros(0, np.int32)
    got = O.encode_graph(model, W, op, dense, none, none, np.zeros((0, 3)), np.zeros(1))
    assert all(np.all(a == 0) for a in got["agg"]) and np.all(got["a0"] == 0)
    rows = []
    for i in range(5):                        # each node alone through the per-node chain
        x = np.concatenate([np.zeros(3), np.eye(5)[op[i]], dense[i]])
        h = relu(relu(x @ W["embed.W0"] + W["embed.b0"]) @ W["embed.W1"] + W["embed.b1"])
        for r in range(2):
            t = np.concatenate([h, np.zeros(8)])
            h = relu(relu(t @ W[f"node{r}.W0"] + W[f"node{r}.b0"]) @ W[f"node{r}.W1"] + W[f"node{r}.b1"])
        rows.append(h)
    t = np.concatenate([np.sum(rows, axis=0), np.zeros(1)])
    u = relu(relu(t @ W["readout.W0"] + W["readout.b0"]) @ W["readout.W1"] + W["readout.b1"])
    np.testing.assert_allclose(got["emb"], u, rtol=1e-12)
    empty = O.encode_graph(model, W, np.zeros(0, np.int32), np.zeros((0, 2)), none, none,
                           np.zeros((0, 3)), np.zeros(1))
    u0 = relu(relu(W["readout.b0"]) @ W["readout.W1"] + W["readout.b1"])
    np.testing.assert_allclose(empty["emb"], u0, rtol=1e-13)
    for ro in ("sum", "mean"):
        m2 = tiny_model(readout=ro)
        assert np.all(O.encode_graph(m2, W, np.zeros(0, np.int32), np.zeros((0, 2)), none, none,
                                     np.zeros((0, 3)), np.zeros(1))["pool"] == 0)


# ------------------------------------------------------------------ P4, P5, P10
def test_relabelling_and_edge_order_invariance():
    rng = np.random.default_rng(6)
    model = tiny_model(rounds=3)
    W = O.unflatten(model, rand_weights(rng, model))
    op, dense, src, dst, xe = rand_graph(rng, model, 10, 24)
    ref = O.encode_graph(model, W, op, dense, src, dst, xe, np.zeros(1))["emb"]
    perm = rng.permutation(10)                # new id of old node i is perm[i]
    inv = np.argsort(perm)
    ep = rng.permutation(24)
    got = O.encode_graph(model, W, op[inv], dense[inv], perm[src][ep].astype(np.int32),
                         perm[dst][ep].astype(np.int32), xe[ep], np.zeros(1))["emb"]
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_duplicated_edges_double_the_sums():
    rng = np.random.default_rng(7)
    model = tiny_model(rounds=1)
    Wd = O.unflatten(model, rand_weights(rng, model))
    Wd["embed.W0"] = Wd["embed.W0"].copy(); Wd["embed.W0"][:3] = 0.0   # h0 ignores edge sums
    op, dense, src, dst, xe = rand_graph(rng, model, 8, 14)
    a = O.encode_graph(model, Wd, op, dense, src, dst, xe, np.zeros(1))
    b = O.encode_graph(model, Wd, op, dense, np.tile(src, 2), np.tile(dst, 2), np.tile(xe, (2, 1)), np.zeros(1))
    np.testing.assert_allclose(b["a0"], 2 * a["a0"], rtol=1e-13)
    np.testing.assert_allclose(b["agg"][0], 2 * a["agg"][0], rtol=1e-13)
    assert np.abs(a["agg"][0]).max() > 0


def test_batch_independence_and_candidate_permutation():
    rng = np.random.default_rng(8)
    model = tiny_model()
    w = rand_weights(rng, model)
    graphs = [rand_graph(rng, model, int(rng.integers(1, 12)), int(rng.integers(0, 20))) for _ in range(7)]
    mask = np.array([1, 1, 0, 1, 1, 1, 0], np.uint8)
    st = state_of(model, graphs, [7], mask)
    emb = O.encode(model, w, st)
    for g in range(7):
        alone = O.encode(model, w, state_of(model, [graphs[g]], [1]))
        assert np.array_equal(alone[0], emb[g])
    pv = O.policy_value(model, w, emb, st)
    order = np.concatenate([[0], 1 + rng.permutation(6)])
    st2 = state_of(model, [graphs[i] for i in order], [7], mask[order])
    pv2 = O.policy_value(model, w, O.encode(model, w, st2), st2)
    np.testing.assert_allclose(pv2["logp"], pv["logp"][order], rtol=1e-12)
    np.testing.assert_allclose(pv2["value"], pv["value"], rtol=1e-12)
    np.testing.assert_allclose(pv2["entropy"], pv["entropy"], rtol=1e-12)


# ------------------------------------------------------------------ P6, P7: softmax identities
def test_masked_softmax_identities():
    rng = np.random.default_rng(9)
    model = tiny_model()
    w = rand_weights(rng, model)
    emb = rng.standard_normal((11, 8))
    mask = np.array([1, 0, 1, 1, 1, 1, 0, 0, 1, 1, 0], np.uint8)
    st = dict(state_graph_ptr=np.array([0, 4, 5, 11], np.int32), slot_mask=mask)
    pv = O.policy_value(model, w, emb, st)
    for s, (a, b) in enumerate([(0, 4), (4, 5), (5, 11)]):
        assert abs(pv["p"][a:b].sum() - 1.0) < 1e-12
        v = np.flatnonzero(mask[a:b]) + a
        l = pv["logit"][v]
        np.testing.assert_allclose(pv["p"][v], np.exp(l) / np.exp(l).sum(), rtol=1e-12)
        assert pv["action"][s] == v[np.argmax(l)] - a
        np.testing.assert_allclose(pv["value"][s],
                                   O.mlp_forward(emb[v].mean(0)[None], O._layers(O.unflatten(model, w), "value"), False)[0][0, 0])
    assert np.all(pv["p"][mask == 0] == 0.0) and np.all(np.isneginf(pv["logp"][mask == 0]))
    assert pv["logp"][4] == 0.0 and pv["entropy"][1] == 0.0 and pv["action"][1] == 0
    # shift invariance: adding a constant to every logit (last bias) leaves logp unchanged
    Wd = O.unflatten(model, w)
    Wd["policy.b2"] = Wd["policy.b2"] + 3.7
    pv2 = O.policy_value(model, O.flatten(model, Wd), emb, st)
    v = mask == 1
    np.testing.assert_allclose(pv2["logp"][v], pv["logp"][v], rtol=1e-12, atol=1e-12)
    # zero last layer: uniform over valid slots, entropy log|V|, ties -> lowest index (No-Op)
    Wd["policy.W2"] = np.zeros_like(Wd["policy.W2"])
    pv3 = O.policy_value(model, O.flatten(model, Wd), emb, st)
    np.testing.assert_allclose(pv3["p"][:4][mask[:4] == 1], 1 / 3, rtol=1e-13)
    np.testing.assert_allclose(pv3["entropy"], np.log([3, 1, 3]), rtol=1e-13, atol=1e-15)
    assert np.all(pv3["action"] == [0, 0, 0])


def test_first_valid_argmax_skips_masked_maximum():
    model = tiny_model()
    rng = np.random.default_rng(10)
    w = rand_weights(rng, model)
    emb = rng.standard_normal((6, 8))
    st = dict(state_graph_ptr=np.array([0, 6], np.int32), slot_mask=np.ones(6, np.uint8))
    full = O.policy_value(model, w, emb, st)
    top = int(np.argmax(full["logit"]))
    if top == 0:
        emb = emb[::-1].copy(); full = O.policy_value(model, w, emb, st); top = int(np.argmax(full["logit"]))
    st["slot_mask"][top] = 0
    pv = O.policy_value(model, w, emb, st)
    l = full["logit"].copy(); l[top] = -np.inf
    assert pv["action"][0] == int(np.argmax(l)) != top


def test_duplicate_of_current_graph_gets_noop_probability():
    rng = np.random.default_rng(11)
    model = tiny_model()
    w = rand_weights(rng, model)
    g0, g1 = rand_graph(rng, model, 9, 14), rand_graph(rng, model, 6, 7)
    st = state_of(model, [g0, g1, g0], [3])
    pv = O.policy_value(model, w, O.encode(model, w, st), st)
    assert pv["logp"][0] == pv["logp"][2] and pv["action"][0] in (0, 1)


# ------------------------------------------------------------------ P11: adjoint identities
def test_gather_and_segment_sum_are_adjoint():
    rng = np.random.default_rng(12)
    n, e, H = 9, 31, 5
    src, dst = rng.integers(0, n, e), rng.integers(0, n, e)
    m, da = rng.standard_normal((e, H)), rng.standard_normal((n, H))
    h, dm = rng.standard_normal((n, H)), rng.standard_normal((e, H))
    assert abs((O.segment_sum(m, dst, n) * da).sum() - (m * da[dst]).sum()) < 1e-12
    assert abs((h[src] * dm).sum() - (h * O.segment_sum(dm, src, n)).sum()) < 1e-12
    D = np.zeros((n, e)); D[dst, np.arange(e)] = 1
    np.testing.assert_allclose(O.segment_sum(m, dst, n), D @ m, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ P8, P9: gradients
def fd_case(seed, readout="sum", round_kind="mlp"):
    rng = np.random.default_rng(seed)
    model = tiny_model(readout=readout, round_kind=round_kind)
    w = rand_weights(rng, model)
    graphs = [rand_graph(rng, model, int(rng.integers(2, 12)), int(rng.integers(1, 22))) for _ in range(7)]
    mask = np.array([1, 1, 0, 1, 1, 0, 1], np.uint8)
    st = state_of(model, graphs, [4, 3], mask)
    st["graph_global"] = rng.standard_normal((7, 1))
    c = rng.standard_normal(7); d = rng.standard_normal(2); f = rng.standard_normal(2)
    return model, w, st, c, d, f


def loss_only(model, w, st, c, d, f):
    pv = O.policy_value(model, w, O.encode(model, w, st), st)
    v = st["slot_mask"] == 1
    return (c[v] * pv["logp"][v]).sum() + (d * pv["value"]).sum() + (f * pv["entropy"]).sum()


@pytest.mark.parametrize("seed,readout,round_kind", [(20, "sum", "mlp"), (21, "mean", "mlp"), (22, "sum", "mlp"),
                                                     (26, "sum", "gat"), (27, "mean", "gat")])
def test_backward_matches_central_differences(seed, readout, round_kind):
    model, w, st, c, d, f = fd_case(seed, readout, round_kind)
    L, grad, _ = O.loss_and_grad(model, w, st, c, d, f)
    assert abs(L - loss_only(model, w, st, c, d, f)) < 1e-12
    rng = np.random.default_rng(seed + 100)
    o, worst = 0, 0.0
    for name, shape in O.weight_layout(model):
        size = int(np.prod(shape))
        for k in rng.choice(size, size=min(size, 64), replace=False):
            i = o + int(k)
            step = 1e-6 * max(1.0, abs(w[i]))
            wp, wm = w.copy(), w.copy()
            wp[i] += step; wm[i] -= step
            fd = (loss_only(model, wp, st, c, d, f) - loss_only(model, wm, st, c, d, f)) / (2 * step)
            err = abs(fd - grad[i]) / max(1e-3, abs(fd), abs(grad[i]))
            worst = max(worst, err)
            assert err < 2e-6, (name, int(k), fd, grad[i])
        o += size
    for _ in range(8):                         # directional derivatives over all weights
        v = rng.standard_normal(w.size); v /= np.linalg.norm(v)
        t = 1e-6
        fd = (loss_only(model, w + t * v, st, c, d, f) - loss_only(model, w - t * v, st, c, d, f)) / (2 * t)
        assert abs(fd - grad @ v) <= 2e-6 * max(1.0, abs(fd))
    assert np.abs(grad).max() > 1e-3


def test_absolute_term_bound_dominates_gradient():
    """The optional bound is the same sum with every term replaced by its absolute value: it
    dominates |grad| entry by entry and equals it where all terms share a sign (last-layer bias
    of the value head: d value / d b = sum of d_s, here made all positive)."""
    model, w, st, c, d, f = fd_case(25)
    b = O.zero_grads(model)
    _, g, _ = O.loss_and_grad(model, w, st, c, np.abs(d), f, bound=b)
    B = O.flatten(model, b)
    assert np.all(B >= np.abs(g) * (1 - 1e-12)) and np.all(B >= 0)
    np.testing.assert_allclose(b["value.b2"], np.abs(d).sum(), rtol=1e-13)
    np.testing.assert_allclose(b["value.b2"], O.unflatten(model, g)["value.b2"], rtol=1e-13)


def test_masked_slots_get_exactly_zero_gradient():
    model, w, st, c, d, f = fd_case(23)
    emb = O.encode(model, w, st)
    demb, gh = O.policy_value_backward(model, w, emb, st, c, d, f)
    masked = st["slot_mask"] == 0
    assert np.all(demb[masked] == 0.0) and np.abs(demb[~masked]).min() > 0
    c2 = c.copy(); c2[masked] = 1e9            # upstream grads on masked slots are ignored
    demb2, gh2 = O.policy_value_backward(model, w, emb, st, c2, d, f)
    assert np.array_equal(demb, demb2) and np.array_equal(gh, gh2)
    # changing a masked candidate's graph changes neither the loss nor the gradient
    L1, g1, _ = O.loss_and_grad(model, w, st, c, d, f)
    st2 = dict(st); st2["edge_feat"] = st["edge_feat"].copy()
    e0, e1 = st["graph_edge_ptr"][2], st["graph_edge_ptr"][3]
    st2["edge_feat"][e0:e1] += 1.0
    L2, g2, _ = O.loss_and_grad(model, w, st2, c, d, f)
    assert L1 == L2 and np.array_equal(g1, g2)


def test_demb_matches_central_differences_on_embeddings():
    model, w, st, c, d, f = fd_case(24)
    emb = O.encode(model, w, st)
    demb, _ = O.policy_value_backward(model, w, emb, st, c, d, f)
    def L(e):
        pv = O.policy_value(model, w, e, st); v = st["slot_mask"] == 1
        return (c[v] * pv["logp"][v]).sum() + (d * pv["value"]).sum() + (f * pv["entropy"]).sum()
    for g in range(7):
        for k in range(8):
            ep, em = emb.copy(), emb.copy()
            ep[g, k] += 1e-6; em[g, k] -= 1e-6
            fd = (L(ep) - L(em)) / 2e-6
            assert abs(fd - demb[g, k]) < 2e-6 * max(1.0, abs(fd))


# ------------------------------------------------------------------ graph-attention reading
def test_attention_round_uniform_case_and_normalisation():
    """Zero attention vectors: alpha = 1/(in-degree + 1) and the round is
    ReLU(D^-1 (A + I) H W), the dense normalised-adjacency product."""
    rng = np.random.default_rng(30)
    model = tiny_model(round_kind="gat", rounds=2)
    w = rand_weights(rng, model)
    Wd = O.unflatten(model, w)
    op, dense, src, dst, xe = rand_graph(rng, model, 9, 20)
    out = O.encode_graph(model, Wd, op, dense, src, dst, xe, np.zeros(1))
    for r in range(2):                        # attention weights of every receiver sum to one
        tot = out["gat"][r]["alpha_s"] + O.segment_sum(out["gat"][r]["alpha_e"], dst, 9)
        np.testing.assert_allclose(tot, 1.0, rtol=1e-13)
    for r in range(2):
        Wd[f"gat{r}.a_src"] = np.zeros(8); Wd[f"gat{r}.a_dst"] = np.zeros(8)
    out = O.encode_graph(model, Wd, op, dense, src, dst, xe, np.zeros(1))
    A = np.eye(9)
    for s, d in zip(src, dst):
        A[d, s] += 1.0
    Hm = out["h"][0]
    for r in range(2):
        Hm = relu((A / A.sum(axis=1, keepdims=True)) @ Hm @ Wd[f"gat{r}.W"])
        np.testing.assert_allclose(out["h"][r + 1], Hm, rtol=1e-12, atol=1e-13)


def test_attention_round_brute_force_softmax():
    rng = np.random.default_rng(31)
    model = tiny_model(round_kind="gat", rounds=1)
    Wd = O.unflatten(model, rand_weights(rng, model))
    op, dense, src, dst, xe = rand_graph(rng, model, 6, 13)
    out = O.encode_graph(model, Wd, op, dense, src, dst, xe, np.zeros(1))
    h0, Wg, a_s, a_d = out["h"][0], Wd["gat0.W"], Wd["gat0.a_src"], Wd["gat0.a_dst"]
    lk = lambda t: t if t > 0 else 0.2 * t
    for i in range(6):
        nbrs = [int(s) for s, d in zip(src, dst) if d == i] + [i]
        z = {j: h0[j] @ Wg for j in set(nbrs)}
        sc = np.array([lk(a_s @ z[j] + a_d @ z[i]) for j in nbrs])
        al = np.exp(sc) / np.exp(sc).sum()
        ref = relu(sum(a * z[j] for a, j in zip(al, nbrs)))
        np.testing.assert_allclose(out["h"][1][i], ref, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ layout / constants
def test_weight_layout_counts_and_paper_constants():
    m = O.default_model(hidden=256, rounds=5)
    assert m["head_hidden"] == (256, 64) and m["rounds"] == 5            # appendix table
    H, De, Dn = 256, 8, 36
    per_round = (2 * H + De) * H + H + H * H + H + 2 * H * H + H + H * H + H
    heads = 2 * (H * 256 + 256 + 256 * 64 + 64 + 64 + 1)
    total = (De + Dn) * H + H + H * H + H + 5 * per_round + (H + 1) * H + H + H * H + H + heads
    assert O.weight_count(m) == total
    names = [n for n, _ in O.weight_layout(m)]
    assert names[0] == "embed.W0" and names[-1] == "value.b2" and len(set(names)) == len(names)


def test_synthetic_configs_are_valid_states():
    for cfg in (1, 2):
        model, st = synth.make_config(cfg)
        gnp, gep = st["graph_node_ptr"], st["graph_edge_ptr"]
        for g in range(len(gnp) - 1):
            n = gnp[g + 1] - gnp[g]
            e = slice(gep[g], gep[g + 1])
            assert n > 0 and st["edge_src"][e].max() < n and st["edge_dst"][e].max() < n
            assert st["edge_src"][e].min() >= 0
        assert np.all(st["slot_mask"][st["state_graph_ptr"][:-1]] == 1)
        m2, st2 = synth.make_config(cfg)
        assert all(np.array_equal(st[k], st2[k]) for k in st if k != "n_states")


# ----------------------------------------------------------------------------- PPO objective
def _ppo_case(rng, S=7, eps=0.2):
    sizes = rng.integers(1, 6, S)
    sgp = np.concatenate([[0], np.cumsum(sizes)])
    G = int(sgp[-1])
    logit = rng.standard_normal(G)
    logp = np.concatenate([l - np.log(np.exp(l).sum()) for l in np.split(logit, sgp[1:-1])])
    action = np.array([rng.integers(0, n) for n in sizes])
    state = dict(state_graph_ptr=sgp)
    return state, logp, rng.standard_normal(S), rng.random(S), action, sizes


def test_ppo_objective_closed_forms():
    """Section 3.3.4's objective at points where its value is known in closed form."""
    rng = np.random.Generator(np.random.PCG64(41))
    state, logp, value, entropy, action, sizes = _ppo_case(rng)
    S = len(sizes)
    slot = state["state_graph_ptr"][:-1] + action
    A, vt = rng.standard_normal(S), rng.standard_normal(S)
    # same policy as the one that sampled (ratio = 1): L_clip = -mean A, gradient -A / S
    r = O.ppo_objective(logp, value, entropy, state, action, logp[slot], A, vt, eps=0.2, c1=0.5, c2=0.01)
    assert abs(r["l_clip"] + A.mean()) < 1e-14
    assert np.allclose(r["dlogp"][slot], -A / S) and np.count_nonzero(r["dlogp"]) <= S
    assert abs(r["l_vf"] - np.mean((value - vt) ** 2)) < 1e-14 and abs(r["l_ent"] + entropy.mean()) < 1e-14
    assert abs(r["J"] - (r["l_clip"] + 0.5 * r["l_vf"] + 0.01 * r["l_ent"])) < 1e-14
    # far outside the clip range: positive advantage and ratio > 1 + eps (or negative and ratio < 1 - eps)
    # gives the clipped constant and no policy gradient; the opposite signs stay unclipped
    old = logp[slot] - np.log(3.0)                                    # ratio = 3
    r = O.ppo_objective(logp, value, entropy, state, action, old, np.abs(A), vt, eps=0.2)
    assert abs(r["l_clip"] + 1.2 * np.abs(A).mean()) < 1e-13 and not r["dlogp"].any()
    r = O.ppo_objective(logp, value, entropy, state, action, old, -np.abs(A), vt, eps=0.2)
    assert abs(r["l_clip"] - 3.0 * np.abs(A).mean()) < 1e-13
    assert np.allclose(r["dlogp"][slot], 3.0 * np.abs(A) / S)
    old = logp[slot] + np.log(4.0)                                    # ratio = 1/4
    r = O.ppo_objective(logp, value, entropy, state, action, old, -np.abs(A), vt, eps=0.2)
    assert abs(r["l_clip"] - 0.8 * np.abs(A).mean()) < 1e-13 and not r["dlogp"].any()


def test_ppo_objective_gradients_by_finite_differences():
    rng = np.random.Generator(np.random.PCG64(43))
    state, logp, value, entropy, action, sizes = _ppo_case(rng, S=9)
    S = len(sizes)
    slot = state["state_graph_ptr"][:-1] + action
    old = logp[slot] + 0.15 * rng.standard_normal(S)                  # ratios on both sides of the clip range
    A, vt = rng.standard_normal(S), rng.standard_normal(S)
    f = lambda lp, v, e: O.ppo_objective(lp, v, e, state, action, old, A, vt, eps=0.1, c1=0.5, c2=0.01)["J"]
    r = O.ppo_objective(logp, value, entropy, state, action, old, A, vt, eps=0.1, c1=0.5, c2=0.01)
    ratio = np.exp(logp[slot] - old)
    assert (np.abs(ratio - 0.9) > 1e-3).all() and (np.abs(ratio - 1.1) > 1e-3).all()   # away from the kinks
    assert ((ratio > 1.1) | (ratio < 0.9)).any() and ((ratio < 1.1) & (ratio > 0.9)).any()
    h = 1e-6
    for name, x, g in (("logp", logp, r["dlogp"]), ("value", value, r["dvalue"]), ("entropy", entropy, r["dentropy"])):
        for i in range(len(x)):
            xp, xm = x.copy(), x.copy()
            xp[i] += h
            xm[i] -= h
            args = dict(lp=logp, v=value, e=entropy)
            key = {"logp": "lp", "value": "v", "entropy": "e"}[name]
            fd = (f(**{**args, key: xp}) - f(**{**args, key: xm})) / (2 * h)
            assert abs(fd - g[i]) < 1e-8, (name, i, fd, g[i])


def test_ppo_objective_hand_example():
    """tests/golden/ppo_hand_example.txt: two states worked by hand from the three equations."""
    rows = [l.split("#")[0].split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "ppo_hand_example.txt"))]
    vals = {r[0]: [float(x) for x in r[1:]] for r in rows if r}
    state = dict(state_graph_ptr=np.array([0, 2, 5]))
    r = O.ppo_objective(vals["logp"], vals["value"], vals["entropy"], state, [1, 0], vals["old_logp"],
                        vals["advantage"], vals["v_target"], eps=0.2, c1=0.5, c2=0.01)
    assert abs(r["l_clip"] - vals["l_clip"][0]) < 1e-12 and abs(r["l_vf"] - vals["l_vf"][0]) < 1e-12
    assert abs(r["l_ent"] - vals["l_ent"][0]) < 1e-12 and abs(r["J"] - vals["J"][0]) < 1e-12
    assert np.allclose(r["dlogp"], vals["dlogp"], atol=1e-12) and np.allclose(r["dvalue"], vals["dvalue"], atol=1e-12)


# ------------------------------------------------------------------ featurisation (Section 3.3.2)
def _shape_examples():
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "shape_features_example.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            t = line.split()
            r = int(t[0])
            rows.append(([int(x) for x in t[1:1 + r]], [float(x) for x in t[1 + r:1 + r + 4]]))
    return rows


def test_shape_features_match_the_printed_example():
    """The paper's example shape and hand-worked padded cases (tests/golden/shape_features_example.txt);
    every extent of the values used is a multiple of a power of two, so the quotients are exact."""
    rows = _shape_examples()
    got = O.edge_features_from_shapes([r[0] for r in rows])
    assert got.shape == (len(rows), 4)
    np.testing.assert_array_equal(got, np.array([r[1] for r in rows]))
    # padding sits on the leading side: the last rank entries are the shape, in order
    assert np.array_equal(O.edge_features_from_shapes([[5, 7]], M=1.0), [[0, 0, 5, 7]])
