"""Host-only checks of xrl_pack_state_edits: states whose candidates are edits of the current graph
(Section 3.3.2: a candidate is the current graph with one rewrite applied) pack to exactly the
arrays xrl_pack_state builds from the candidate graphs written out in full; bad edits are rejected
with the documented error codes."""
import numpy as np
import pytest

import paper_2304_14698_amd as xrl
import synth
from test_host_pack import base_model


def views_equal(a, b):
    va, vb = a.host_view(), b.host_view()
    assert (a.S, a.G, a.N, a.E) == (b.S, b.G, b.N, b.E)
    assert set(va) == set(vb)
    for k in va:
        np.testing.assert_array_equal(va[k], vb[k], err_msg=k)


@pytest.mark.parametrize("shape,n_states,n_cand", [("layered", 1, 8), ("transformer", 1, 24), ("inception", 3, 5),
                                                  ("layered", 4, 0)])
def test_edit_pack_equals_full_pack(shape, n_states, n_cand):
    rng = np.random.Generator(np.random.PCG64(314 + n_cand))
    make = dict(layered=lambda: synth.layered_dag(rng, 60), transformer=lambda: synth.transformer_dag(rng, 4),
                inception=lambda: synth.inception_dag(rng, 3))[shape]
    bases = [synth.shuffle_edges(rng, make()) for _ in range(n_states)]
    edit_state, state = synth.make_edit_states(rng, bases, n_cand, by_block=shape != "layered")
    m = base_model()
    full = xrl.pack_state(m, state)
    ed = xrl.pack_state_edits(m, edit_state)
    views_equal(ed, full)
    full.free()
    ed.free()


def extreme_edit_state():
    """Candidates that delete all but one node, delete every edge, only add, add nothing, add an
    isolated node, and a new node that is a hub of 40 in-edges (a receiver split over two edge
    tiles); candidate counts differing per state."""
    rng = np.random.Generator(np.random.PCG64(99))
    g = synth.shuffle_edges(rng, synth.layered_dag(rng, 50))
    n, e = g.n_nodes, g.n_edges
    none = dict(del_node=np.zeros(0, np.int32), del_edge=np.zeros(0, np.int32), add_node_op=np.zeros(0, np.int32),
                add_node_dense=np.zeros((0, 4), np.float32), add_edge_src=np.zeros(0, np.int32),
                add_edge_dst=np.zeros(0, np.int32), add_edge_feat=np.zeros((0, 8), np.float32))
    f = lambda k: rng.standard_normal((k, 8)).astype(np.float32)
    eds = [
        dict(none),
        dict(none, del_node=np.arange(1, n, dtype=np.int32)),
        dict(none, del_edge=np.arange(e, dtype=np.int32)),
        dict(none, add_node_op=np.array([3], np.int32), add_node_dense=np.ones((1, 4), np.float32)),
        dict(none, add_node_op=np.array([5, 6], np.int32), add_node_dense=np.zeros((2, 4), np.float32),
             add_edge_src=np.array([0, n, n + 1, 2], np.int32), add_edge_dst=np.array([n, n + 1, 4, 2], np.int32),
             add_edge_feat=f(4)),
        dict(none, del_node=np.array([0, 7], np.int32), add_node_op=np.array([9], np.int32),
             add_node_dense=np.full((1, 4), 2, np.float32),
             add_edge_src=np.concatenate([np.arange(1, 7), np.arange(8, 42)]).astype(np.int32),
             add_edge_dst=np.full(40, n, np.int32), add_edge_feat=f(40)),
    ]
    graphs = [g] + [synth.apply_edit(g, ed) for ed in eds]
    g2 = synth.layered_dag(rng, 10)
    mask = np.ones(len(graphs), np.uint8)
    mask[2] = 0
    state = synth.concat_states([(graphs, mask), ([g2], np.ones(1, np.uint8))])
    ptr = lambda key: np.concatenate([[0], np.cumsum([len(ed[key]) for ed in eds])]).astype(np.int32)
    cat = lambda key: np.concatenate([ed[key] for ed in eds])
    edit_state = dict(
        n_states=2, cur_node_ptr=np.array([0, n, n + g2.n_nodes], np.int32), cur_edge_ptr=np.array([0, e, e + g2.n_edges], np.int32),
        node_op=np.concatenate([g.op, g2.op]), node_dense=np.concatenate([g.dense, g2.dense]),
        edge_src=np.concatenate([g.src, g2.src]), edge_dst=np.concatenate([g.dst, g2.dst]),
        edge_feat=np.concatenate([g.efeat, g2.efeat]), state_cand_ptr=np.array([0, len(eds), len(eds)], np.int32),
        del_node_ptr=ptr("del_node"), del_node=cat("del_node"), del_edge_ptr=ptr("del_edge"), del_edge=cat("del_edge"),
        add_node_ptr=ptr("add_node_op"), add_node_op=cat("add_node_op"), add_node_dense=cat("add_node_dense"),
        add_edge_ptr=ptr("add_edge_src"), add_edge_src=cat("add_edge_src"), add_edge_dst=cat("add_edge_dst"),
        add_edge_feat=cat("add_edge_feat"), graph_global=state["graph_global"], slot_mask=state["slot_mask"])
    return edit_state, state


def test_edit_pack_extreme_edits():
    edit_state, state = extreme_edit_state()
    m = base_model()
    full = xrl.pack_state(m, state)
    ed = xrl.pack_state_edits(m, edit_state)
    views_equal(ed, full)
    assert full.host_view()["tile_ptr"].size > 2


def test_edit_pack_rejects_bad_edits():
    good, _ = extreme_edit_state()
    m = base_model()
    n = int(good["cur_node_ptr"][1])

    def expect(code, **kw):
        st = dict(good)
        for k, v in kw.items():
            st[k] = v
        with pytest.raises(xrl.XrlError) as ei:
            xrl.pack_state_edits(m, st)
        assert ei.value.code == xrl.ERR[code], (kw.keys(), ei.value)

    dn = good["del_node"].copy(); dn[0] = n                       # deleted node out of range
    expect("INDEX", del_node=dn)
    dn = good["del_node"].copy(); dn[1], dn[2] = dn[2], dn[1]     # not ascending
    expect("INDEX", del_node=dn)
    de = good["del_edge"].copy(); de[3] = de[2]                   # repeated edge
    expect("INDEX", del_edge=de)
    s = good["add_edge_src"].copy(); s[-1] = 0                    # the last candidate deleted node 0
    expect("INDEX", add_edge_src=s)
    d = good["add_edge_dst"].copy(); d[0] = n + 5                 # beyond the candidate's new nodes
    expect("INDEX", add_edge_dst=d)
    op = good["add_node_op"].copy(); op[0] = 32
    expect("INDEX", add_node_op=op)
    f = good["add_edge_feat"].copy(); f[2, 1] = np.inf
    expect("VALUE", add_edge_feat=f)
    mk = good["slot_mask"].copy(); mk[0] = 0
    expect("MASK", slot_mask=mk)
    p = good["add_edge_ptr"].copy(); p[2] = p[1] - 1 if p[1] > 0 else 5
    p[1] = 5
    expect("SHAPE", add_edge_ptr=p)
    expect("NULL", del_node=None)
