"""States (current graph + candidate graphs + slot mask) in the flat array layout the packer
takes, the five benchmark configurations, weight initialisation and upstream gradients."""
import numpy as np
from . import graphs as G

BASE_SEED = 230414698

# name, base-graph builder, candidates per state, rewrite size, #states, model dims, precision
CONFIGS = {
    1: dict(name="tiny", base="layered", n_cand=8, touch=None, del_ins=(1, 4), by_block=False,
            n_states=1, hidden=64, rounds=2, precision="fp32"),
    2: dict(name="transformer", base="transformer12", n_cand=128, touch=(1, 6), by_block=True,
            n_states=1, hidden=128, rounds=5, precision="bf16"),
    3: dict(name="resnet50x32", base="resnet", n_cand=64, touch=(1, 6), by_block=True,
            n_states=32, hidden=128, rounds=5, precision="bf16"),
    4: dict(name="inceptionv3", base="inception", n_cand=256, touch=(1, 6), by_block=True,
            n_states=1, hidden=256, rounds=5, precision="bf16"),
    5: dict(name="ppo_minibatch", base="transformer20", n_cand=(64, 512), touch=(1, 6),
            by_block=True, n_states=64, hidden=256, rounds=5, precision="bf16"),
}


def _base_graph(rng, kind):
    if kind == "layered":
        return G.layered_dag(rng, 50)
    if kind == "transformer12":
        return G.transformer_dag(rng, 12)
    if kind == "transformer20":
        return G.transformer_dag(rng, 20)
    if kind == "resnet":
        return G.resnet_dag(rng, 16)
    if kind == "inception":
        return G.inception_dag(rng, 11)
    raise ValueError(kind)


def make_state(rng, base, n_cand, touch=(1, 6), del_ins=None, by_block=True, mask_p=0.1):
    """One state: slot 0 = the current graph (the No-Op slot, always valid), slots 1..n_cand =
    local rewrites of it; each candidate slot is masked out independently with prob. mask_p.
    Returns a list of Graph and a uint8 mask."""
    graphs = [G.shuffle_edges(rng, base)]
    for _ in range(n_cand):
        if del_ins is not None:
            nd = int(rng.integers(del_ins[0], del_ins[1] + 1))
            ni = int(rng.integers(del_ins[0], del_ins[1] + 1))
        else:
            t = int(rng.integers(touch[0], touch[1] + 1))
            nd = int(rng.integers(0, t + 1))
            ni = t - nd
        graphs.append(G.local_rewrite(rng, base, nd, ni, by_block=by_block))
    mask = (rng.random(n_cand + 1) >= mask_p).astype(np.uint8)
    mask[0] = 1
    return graphs, mask


def concat_states(states, d_global=1):
    """List of (graphs, mask) -> dict of flat arrays (edge endpoints stay graph-local)."""
    gl = [g for graphs, _ in states for g in graphs]
    sgp = np.zeros(len(states) + 1, dtype=np.int32)
    sgp[1:] = np.cumsum([len(graphs) for graphs, _ in states])
    gnp = np.zeros(len(gl) + 1, dtype=np.int32)
    gnp[1:] = np.cumsum([g.n_nodes for g in gl])
    gep = np.zeros(len(gl) + 1, dtype=np.int32)
    gep[1:] = np.cumsum([g.n_edges for g in gl])
    return dict(
        n_states=len(states),
        state_graph_ptr=sgp, graph_node_ptr=gnp, graph_edge_ptr=gep,
        node_op=np.concatenate([g.op for g in gl]).astype(np.int32),
        node_dense=np.concatenate([g.dense for g in gl]).astype(np.float32),
        edge_src=np.concatenate([g.src for g in gl]).astype(np.int32),
        edge_dst=np.concatenate([g.dst for g in gl]).astype(np.int32),
        edge_feat=np.concatenate([g.efeat for g in gl]).astype(np.float32),
        graph_global=np.zeros((len(gl), d_global), dtype=np.float32),
        slot_mask=np.concatenate([m for _, m in states]).astype(np.uint8),
    )


def state_subset(state, states_idx):
    """Sub-batch holding only the listed states (whole states, all their graphs)."""
    sgp, gnp, gep = state["state_graph_ptr"], state["graph_node_ptr"], state["graph_edge_ptr"]
    gsel = np.concatenate([np.arange(sgp[s], sgp[s + 1]) for s in states_idx])
    nsel = np.concatenate([np.arange(gnp[g], gnp[g + 1]) for g in gsel])
    esel = np.concatenate([np.arange(gep[g], gep[g + 1]) for g in gsel])
    out = dict(n_states=len(states_idx))
    out["state_graph_ptr"] = np.concatenate(
        [[0], np.cumsum([sgp[s + 1] - sgp[s] for s in states_idx])]).astype(np.int32)
    out["graph_node_ptr"] = np.concatenate(
        [[0], np.cumsum(gnp[gsel + 1] - gnp[gsel])]).astype(np.int32)
    out["graph_edge_ptr"] = np.concatenate(
        [[0], np.cumsum(gep[gsel + 1] - gep[gsel])]).astype(np.int32)
    for k in ("node_op", "node_dense"):
        out[k] = state[k][nsel]
    for k in ("edge_src", "edge_dst", "edge_feat"):
        out[k] = state[k][esel]
    out["graph_global"] = state["graph_global"][gsel]
    out["slot_mask"] = state["slot_mask"][gsel]
    return out


def make_config(cfg, rep=0, n_states=None, n_cand=None):
    """The synthetic meta-batch of configuration `cfg` (1..5). n_states / n_cand override the
    configured counts (used for reduced-size test cases). Returns (model dict, state dict)."""
    c = CONFIGS[cfg]
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * cfg + rep))
    base = _base_graph(rng, c["base"])
    S = c["n_states"] if n_states is None else n_states
    states = []
    for _ in range(S):
        nc = c["n_cand"] if n_cand is None else n_cand
        if isinstance(nc, tuple):
            nc = int(rng.integers(nc[0], nc[1] + 1))
        states.append(make_state(rng, base, nc, touch=c["touch"], del_ins=c.get("del_ins"),
                                 by_block=c["by_block"]))
    model = dict(n_op_types=G.N_OP_TYPES, n_node_dense=G.N_NODE_DENSE, d_edge=G.D_EDGE,
                 d_global=1, hidden=c["hidden"], rounds=c["rounds"], mlp_layers=2,
                 head_hidden=(256, 64), readout="sum", precision=c["precision"])
    return model, concat_states(states)


def init_weights(rng, layout, bias_range=0.1):
    """Flat fp32 weight vector for a layout = list of (name, shape): matrices (2-D, [in, out])
    Glorot-uniform, vectors uniform in +-bias_range (0 gives zero biases)."""
    parts = []
    for _, shape in layout:
        if len(shape) == 2:
            a = np.sqrt(6.0 / (shape[0] + shape[1]))
            parts.append(rng.uniform(-a, a, size=shape).astype(np.float32).ravel())
        else:
            parts.append(rng.uniform(-bias_range, bias_range, size=shape).astype(np.float32).ravel())
    return np.concatenate(parts)


def upstream_grads(rng, n_graphs, n_states):
    """Seeded upstream gradients of a scalar loss w.r.t. (logp, value, entropy): N(0,1)/G."""
    s = 1.0 / max(n_graphs, 1)
    return ((rng.standard_normal(n_graphs) * s).astype(np.float32),
            (rng.standard_normal(n_states) * s).astype(np.float32),
            (rng.standard_normal(n_states) * s).astype(np.float32))


def random_states(rng, model, n_states, max_graphs=6, max_nodes=120, edge_factor=(0.0, 2.5), mask_p=0.25):
    """Unstructured random states for robustness sweeps: every state has 1..max_graphs graphs of
    0..max_nodes nodes and a random number of arbitrary edges (self loops and repeated edges
    included, any direction), random attributes, random slot masks (slot 0 always valid)."""
    De, Dd, Dg, T = model["d_edge"], model["n_node_dense"], model["d_global"], model["n_op_types"]
    ns, es, srcs, dsts, sgp, mask = [], [], [], [], [0], []
    for _ in range(n_states):
        g_s = int(rng.integers(1, max_graphs + 1))
        for j in range(g_s):
            n = int(rng.integers(0, max_nodes + 1))
            e = int(rng.uniform(*edge_factor) * n) if n > 0 else 0
            ns.append(n); es.append(e)
            srcs.append(rng.integers(0, max(n, 1), e).astype(np.int32))
            dsts.append(rng.integers(0, max(n, 1), e).astype(np.int32))
            mask.append(1 if j == 0 else int(rng.random() >= mask_p))
        sgp.append(sgp[-1] + g_s)
    N, E, G = sum(ns), sum(es), len(ns)
    return dict(n_states=n_states, state_graph_ptr=np.array(sgp, np.int32),
                graph_node_ptr=np.concatenate([[0], np.cumsum(ns)]).astype(np.int32),
                graph_edge_ptr=np.concatenate([[0], np.cumsum(es)]).astype(np.int32),
                node_op=rng.integers(0, T, N).astype(np.int32),
                node_dense=rng.integers(0, 13, (N, Dd)).astype(np.float32),
                edge_src=np.concatenate(srcs + [np.zeros(0, np.int32)]).astype(np.int32),
                edge_dst=np.concatenate(dsts + [np.zeros(0, np.int32)]).astype(np.int32),
                edge_feat=(rng.standard_normal((E, De)) * 0.3).astype(np.float32),
                graph_global=rng.standard_normal((G, Dg)).astype(np.float32),
                slot_mask=np.array(mask, np.uint8))


def make_edit_states(rng, bases, n_cand, touch=(1, 6), by_block=True, mask_p=0.1, n_del_edges=(0, 2)):
    """States whose candidates are edits of the current graph. bases: one current Graph per state;
    n_cand: candidates per state (an int or one per state). Returns (edit_state, state): the dict
    of arrays xrl_pack_state_edits takes, and the ordinary state (every candidate written out as
    the graph its edit stands for) that it must pack identically to."""
    S = len(bases)
    counts = [n_cand] * S if np.isscalar(n_cand) else list(n_cand)
    edits, full = [], []
    for s in range(S):
        g = bases[s]
        graphs, eds = [g], []
        for _ in range(counts[s]):
            t = int(rng.integers(touch[0], touch[1] + 1))
            nd = int(rng.integers(0, t + 1))
            ed = G.local_rewrite_edit(rng, g, nd, t - nd, by_block=by_block,
                                      n_del_edges=int(rng.integers(n_del_edges[0], n_del_edges[1] + 1)))
            eds.append(ed)
            graphs.append(G.apply_edit(g, ed))
        mask = (rng.random(counts[s] + 1) >= mask_p).astype(np.uint8)
        mask[0] = 1
        edits.append(eds)
        full.append((graphs, mask))
    state = concat_states(full)
    flat = [ed for eds in edits for ed in eds]
    ptr = lambda key: np.concatenate([[0], np.cumsum([len(ed[key]) for ed in flat])]).astype(np.int32)
    cat = lambda key, shape, dt: (np.concatenate([ed[key] for ed in flat]) if flat else np.zeros(shape, dt)).astype(dt).reshape((-1,) + shape[1:])
    edit_state = dict(
        n_states=S,
        cur_node_ptr=np.concatenate([[0], np.cumsum([g.n_nodes for g in bases])]).astype(np.int32),
        cur_edge_ptr=np.concatenate([[0], np.cumsum([g.n_edges for g in bases])]).astype(np.int32),
        node_op=np.concatenate([g.op for g in bases]).astype(np.int32),
        node_dense=np.concatenate([g.dense for g in bases]).astype(np.float32),
        edge_src=np.concatenate([g.src for g in bases]).astype(np.int32),
        edge_dst=np.concatenate([g.dst for g in bases]).astype(np.int32),
        edge_feat=np.concatenate([g.efeat for g in bases]).astype(np.float32),
        state_cand_ptr=np.concatenate([[0], np.cumsum(counts)]).astype(np.int32),
        del_node_ptr=ptr("del_node"), del_node=cat("del_node", (0,), np.int32),
        del_edge_ptr=ptr("del_edge"), del_edge=cat("del_edge", (0,), np.int32),
        add_node_ptr=ptr("add_node_op"), add_node_op=cat("add_node_op", (0,), np.int32),
        add_node_dense=cat("add_node_dense", (0, G.N_NODE_DENSE), np.float32),
        add_edge_ptr=ptr("add_edge_src"), add_edge_src=cat("add_edge_src", (0,), np.int32),
        add_edge_dst=cat("add_edge_dst", (0,), np.int32), add_edge_feat=cat("add_edge_feat", (0, G.D_EDGE), np.float32),
        graph_global=state["graph_global"], slot_mask=state["slot_mask"])
    return edit_state, state
