"""Synthetic computation-graph DAGs shaped like DNN graphs, and local-rewrite candidates.

Every function takes a numpy Generator and is deterministic given it. A Graph holds plain
arrays only: op ids, dense node attributes, an unsorted edge list with per-edge attributes,
plus two bookkeeping fields (layer, block) used only to keep rewrites local and acyclic.
"""
from dataclasses import dataclass
import numpy as np

N_OP_TYPES = 32
N_NODE_DENSE = 4
D_EDGE = 8

# op-id table of the synthetic graphs (32 ids; the named ones are used by the templates)
OP = {name: i for i, name in enumerate([
    "input", "weight", "matmul", "add", "softmax", "layernorm", "reshape", "transpose",
    "conv", "batchnorm", "relu", "concat", "pool", "split", "mul", "sigmoid",
    "tanh", "gelu", "dropout", "slice", "pad", "reduce", "squeeze", "unsqueeze",
    "gather", "cast", "div", "sub", "exp", "sqrt", "erf", "identity"])}


@dataclass
class Graph:
    op: np.ndarray       # [n] int32 in [0, 32)
    dense: np.ndarray    # [n, 4] float32, integer-valued in [0, 12]
    layer: np.ndarray    # [n] int32 topological position (edges go from lower to higher)
    block: np.ndarray    # [n] int32 id of the repeated block the node belongs to
    src: np.ndarray      # [e] int32 sender, local node index
    dst: np.ndarray      # [e] int32 receiver, local node index
    efeat: np.ndarray    # [e, 8] float32

    @property
    def n_nodes(self):
        return int(self.op.shape[0])

    @property
    def n_edges(self):
        return int(self.src.shape[0])


def _finish(rng, ops, blocks, edges, op_random=False):
    """Attach features to a topology given as lists (nodes were added in topological order)."""
    n = len(ops)
    src = np.array([e[0] for e in edges], dtype=np.int32).reshape(-1)
    dst = np.array([e[1] for e in edges], dtype=np.int32).reshape(-1)
    layer = np.zeros(n, dtype=np.int32)
    order = np.argsort(dst, kind="stable")
    for k in order:                       # receivers ascending == topological order here
        s, d = src[k], dst[k]
        if layer[s] + 1 > layer[d]:
            layer[d] = layer[s] + 1
    op = (rng.integers(0, N_OP_TYPES, size=n) if op_random else np.array(ops)).astype(np.int32)
    dense = rng.integers(0, 13, size=(n, N_NODE_DENSE)).astype(np.float32)
    efeat = rng.standard_normal((len(edges), D_EDGE)).astype(np.float32)
    return Graph(op, dense, layer, np.array(blocks, dtype=np.int32), src, dst, efeat)


class _Builder:
    def __init__(self):
        self.ops, self.blocks, self.edges, self.blk = [], [], [], 0

    def node(self, name, *inputs):
        i = len(self.ops)
        self.ops.append(OP[name])
        self.blocks.append(self.blk)
        for s in inputs:
            self.edges.append((s, i))
        return i

    def leaf(self, name="weight"):
        return self.node(name)


def layered_dag(rng, n_target=50):
    """Layers of width U{1..4} until about n_target nodes; every node below the first layer
    draws U{1,2} distinct predecessors from the previous three layers; op ids uniform."""
    layers, n = [], 0
    while n < n_target:
        w = int(rng.integers(1, 5))
        layers.append(list(range(n, n + w)))
        n += w
    edges, blocks = [], []
    for li, nodes in enumerate(layers):
        pool = [p for L in layers[max(0, li - 3):li] for p in L]
        for v in nodes:
            blocks.append(li // 4)
            if pool:
                k = min(int(rng.integers(1, 3)), len(pool))
                for p in rng.choice(len(pool), size=k, replace=False):
                    edges.append((pool[int(p)], v))
    g = _finish(rng, [0] * n, blocks, edges, op_random=True)
    # layer index = generation layer (needed for +-3-layer rewiring), not longest path
    lay = np.zeros(n, dtype=np.int32)
    for li, nodes in enumerate(layers):
        lay[nodes] = li
    g.layer = lay
    return g


def transformer_dag(rng, n_blocks=12):
    """Chain of attention + feed-forward blocks (about 48 nodes each) with parameter leaves
    and residual skip edges; op ids from {matmul, add, softmax, layernorm, reshape, transpose}
    plus input/weight leaves."""
    b = _Builder()
    x = b.leaf("input")
    for blk in range(n_blocks):
        b.blk = blk
        ln1 = b.node("layernorm", x, b.leaf(), b.leaf())
        heads = []
        for _ in range(3):                                   # q, k, v projections
            t = b.node("matmul", ln1, b.leaf())
            t = b.node("add", t, b.leaf())
            t = b.node("reshape", t)
            heads.append(b.node("transpose", t))
        q, k, v = heads
        kt = b.node("transpose", k)
        s = b.node("matmul", q, kt)
        s = b.node("add", s, b.leaf())
        p = b.node("softmax", s)
        o = b.node("matmul", p, v)
        o = b.node("reshape", b.node("transpose", o))
        o = b.node("add", b.node("matmul", o, b.leaf()), b.leaf())
        r1 = b.node("add", x, o)
        ln2 = b.node("layernorm", r1, b.leaf(), b.leaf())
        f = b.node("add", b.node("matmul", ln2, b.leaf()), b.leaf())
        f = b.node("reshape", f)
        f = b.node("add", b.node("matmul", f, b.leaf()), b.leaf())
        x = b.node("add", r1, f)
    return _finish(rng, b.ops, b.blocks, b.edges)


def resnet_dag(rng, n_blocks=16):
    """Stem, n_blocks bottleneck residual blocks (conv/batchnorm/relu x3, add with a skip
    edge; every fourth block has a projection on the skip), pooling + classifier head."""
    b = _Builder()

    def cbr(t, relu=True):
        t = b.node("conv", t, b.leaf())
        t = b.node("batchnorm", t, b.leaf(), b.leaf())
        return b.node("relu", t) if relu else t

    x = b.node("pool", cbr(b.leaf("input")))
    for blk in range(n_blocks):
        b.blk = blk + 1
        t = cbr(cbr(cbr(x), True), relu=False)
        skip = cbr(x, relu=False) if blk % 4 == 0 else x
        x = b.node("relu", b.node("add", t, skip))
    b.blk = n_blocks + 1
    x = b.node("reshape", b.node("pool", x))
    b.node("add", b.node("matmul", x, b.leaf()), b.leaf())
    return _finish(rng, b.ops, b.blocks, b.edges)


def inception_dag(rng, n_modules=11):
    """Modules of 4-6 parallel branches (2-4 conv/batchnorm/relu units each) from one
    fan-out node into one concat node: receiver in-degree mostly 1-3 with hubs of 4-6,
    sender out-degree hubs of 4-6."""
    b = _Builder()

    def cbr(t):
        t = b.node("conv", t, b.leaf(), b.leaf())
        t = b.node("batchnorm", t, b.leaf(), b.leaf())
        return b.node("relu", t)

    x = cbr(cbr(b.leaf("input")))
    for m in range(n_modules):
        b.blk = m + 1
        outs = []
        for _ in range(int(rng.integers(4, 7))):
            t = x
            for _ in range(int(rng.integers(2, 5))):
                t = cbr(t)
            outs.append(t)
        x = b.node("concat", *outs)
    b.blk = n_modules + 1
    x = b.node("reshape", b.node("pool", x))
    b.node("add", b.node("matmul", x, b.leaf()), b.leaf())
    return _finish(rng, b.ops, b.blocks, b.edges)


def shuffle_edges(rng, g):
    """Same graph with its edge list in a random order (edge attributes follow)."""
    p = rng.permutation(g.n_edges)
    return Graph(g.op, g.dense, g.layer, g.block, g.src[p], g.dst[p], g.efeat[p])


def local_rewrite(rng, g, n_del, n_ins, by_block=False, reach=3):
    """A candidate graph: copy of g with n_del nodes deleted (their edges dropped) and n_ins
    nodes inserted near a random anchor; each new node is wired to 1-2 predecessors from the
    `reach` layers below its layer and 1-2 successors from the `reach` layers above, so the
    result stays acyclic. Surviving nodes keep their relative order; new nodes come last;
    the edge list is returned in a random order."""
    n = g.n_nodes
    anchor = int(rng.integers(0, n))
    if by_block:
        near = np.flatnonzero(g.block == g.block[anchor])
    else:
        near = np.flatnonzero(np.abs(g.layer - g.layer[anchor]) <= reach)
    n_del = min(n_del, max(len(near) - 1, 0), n - 1)
    dele = rng.choice(near, size=n_del, replace=False) if n_del > 0 else np.zeros(0, np.int64)
    keep = np.ones(n, dtype=bool)
    keep[dele] = False
    newid = np.cumsum(keep, dtype=np.int64) - 1
    ekeep = keep[g.src] & keep[g.dst]
    src = newid[g.src[ekeep]]
    dst = newid[g.dst[ekeep]]
    efeat = g.efeat[ekeep]
    op, dense = g.op[keep], g.dense[keep]
    layer, block = g.layer[keep], g.block[keep]
    nk = int(keep.sum())

    new_src, new_dst = [], []
    nl = np.clip(g.layer[anchor] + rng.integers(-1, 2, size=n_ins), 0, None).astype(np.int32)
    for j in range(n_ins):
        v, L = nk + j, int(nl[j])
        below = np.flatnonzero((layer >= L - reach) & (layer <= L - 1))
        above = np.flatnonzero((layer >= L + 1) & (layer <= L + reach))
        for pool, is_pred in ((below, True), (above, False)):
            if len(pool) == 0:
                continue
            k = min(int(rng.integers(1, 3)), len(pool))
            for u in rng.choice(pool, size=k, replace=False):
                if is_pred:
                    new_src.append(int(u)); new_dst.append(v)
                else:
                    new_src.append(v); new_dst.append(int(u))
    ne = len(new_src)
    op = np.concatenate([op, rng.integers(0, N_OP_TYPES, size=n_ins).astype(np.int32)])
    dense = np.concatenate([dense, rng.integers(0, 13, size=(n_ins, N_NODE_DENSE)).astype(np.float32)])
    layer = np.concatenate([layer, nl])
    block = np.concatenate([block, np.full(n_ins, g.block[anchor], dtype=np.int32)])
    src = np.concatenate([src, np.array(new_src, dtype=np.int64)]).astype(np.int32)
    dst = np.concatenate([dst, np.array(new_dst, dtype=np.int64)]).astype(np.int32)
    efeat = np.concatenate([efeat, rng.standard_normal((ne, D_EDGE)).astype(np.float32)])
    p = rng.permutation(len(src))
    return Graph(op, dense, layer, block, src[p], dst[p], efeat[p])


def local_rewrite_edit(rng, g, n_del, n_ins, by_block=False, reach=3, n_del_edges=0):
    """A candidate as an edit of g (the form a rewrite engine produces): nodes of g that
    disappear, further edges of g that disappear, new nodes, new edges. An endpoint of a new edge
    is a surviving node id of g, or g.n_nodes + k for the k-th new node. Same locality rules as
    local_rewrite. Returns a dict of arrays."""
    n = g.n_nodes
    anchor = int(rng.integers(0, n))
    near = np.flatnonzero(g.block == g.block[anchor]) if by_block else np.flatnonzero(np.abs(g.layer - g.layer[anchor]) <= reach)
    n_del = min(n_del, max(len(near) - 1, 0), n - 1)
    dele = np.sort(rng.choice(near, size=n_del, replace=False)) if n_del > 0 else np.zeros(0, np.int64)
    keep = np.ones(n, dtype=bool)
    keep[dele] = False
    alive_edges = np.flatnonzero(keep[g.src] & keep[g.dst])
    n_del_edges = min(n_del_edges, len(alive_edges))
    dedge = np.sort(rng.choice(alive_edges, size=n_del_edges, replace=False)) if n_del_edges > 0 else np.zeros(0, np.int64)
    nl = np.clip(g.layer[anchor] + rng.integers(-1, 2, size=n_ins), 0, None).astype(np.int32)
    new_src, new_dst = [], []
    for j in range(n_ins):
        v, L = n + j, int(nl[j])
        below = np.flatnonzero(keep & (g.layer >= L - reach) & (g.layer <= L - 1))
        above = np.flatnonzero(keep & (g.layer >= L + 1) & (g.layer <= L + reach))
        for pool, is_pred in ((below, True), (above, False)):
            if len(pool) == 0:
                continue
            k = min(int(rng.integers(1, 3)), len(pool))
            for u in rng.choice(pool, size=k, replace=False):
                if is_pred:
                    new_src.append(int(u)); new_dst.append(v)
                else:
                    new_src.append(v); new_dst.append(int(u))
    ne = len(new_src)
    return dict(del_node=dele.astype(np.int32), del_edge=dedge.astype(np.int32),
                add_node_op=rng.integers(0, N_OP_TYPES, size=n_ins).astype(np.int32),
                add_node_dense=rng.integers(0, 13, size=(n_ins, N_NODE_DENSE)).astype(np.float32),
                add_edge_src=np.array(new_src, dtype=np.int32), add_edge_dst=np.array(new_dst, dtype=np.int32),
                add_edge_feat=rng.standard_normal((ne, D_EDGE)).astype(np.float32))


def apply_edit(g, ed):
    """The candidate graph an edit stands for: surviving nodes of g in their order, then the new
    nodes; surviving edges of g in their order, then the new edges."""
    n = g.n_nodes
    keep = np.ones(n, dtype=bool)
    keep[ed["del_node"]] = False
    n_new = len(ed["add_node_op"])
    newid = np.concatenate([np.cumsum(keep, dtype=np.int64) - 1, int(keep.sum()) + np.arange(n_new)])
    ekeep = keep[g.src] & keep[g.dst]
    ekeep[ed["del_edge"]] = False
    src = np.concatenate([newid[g.src[ekeep]], newid[ed["add_edge_src"]]]).astype(np.int32)
    dst = np.concatenate([newid[g.dst[ekeep]], newid[ed["add_edge_dst"]]]).astype(np.int32)
    return Graph(np.concatenate([g.op[keep], ed["add_node_op"]]).astype(np.int32),
                 np.concatenate([g.dense[keep], ed["add_node_dense"]]).astype(np.float32),
                 np.concatenate([g.layer[keep], np.zeros(n_new, np.int32)]), np.concatenate([g.block[keep], np.zeros(n_new, np.int32)]),
                 src, dst, np.concatenate([g.efeat[ekeep], ed["add_edge_feat"]]).astype(np.float32))
