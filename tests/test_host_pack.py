"""Host-only checks of the C-ABI library: it loads without a GPU, exports every declared symbol,
lays the weights out like the oracle, packs states correctly and rejects bad input with the
documented error codes (never touching the GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2304_14698_amd as xrl
import synth
from oracle import xrl_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def base_model(**kw):
    m = dict(n_op_types=32, n_node_dense=4, d_edge=8, d_global=1, hidden=64, rounds=2, mlp_layers=2,
             head_hidden=(256, 64), readout="sum", precision="fp32")
    m.update(kw)
    return m


def test_library_exports_every_declared_symbol():
    lib = xrl.load_library()
    text = open(os.path.join(ROOT, "include", "xrl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)          # drop comments
    declared = set(re.findall(r"\b(xrl_[a-z_]+)\s*\(", text))
    assert declared == set(xrl.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert b"xrl" in lib.xrl_version()


@pytest.mark.parametrize("kw", [dict(), dict(hidden=256, rounds=5), dict(hidden=128, rounds=0),
                                dict(n_op_types=40, n_node_dense=0, d_edge=4, mlp_layers=1, hidden=64),
                                dict(hidden=128, rounds=3, round_kind="gat")])
def test_weight_layout_matches_oracle(kw):
    m = base_model(**kw)
    om = O.default_model(**{k: m[k] for k in ("n_op_types", "n_node_dense", "d_edge", "d_global",
                                              "hidden", "rounds", "mlp_layers", "head_hidden")},
                         round_kind=m.get("round_kind", "mlp"))
    assert xrl.weight_layout(m) == [(n, tuple(s)) for n, s in O.weight_layout(om)]
    assert xrl.weight_count(m) == O.weight_count(om)


def test_pack_matches_edge_list():
    model, st = synth.make_config(1)
    b = xrl.pack_state(model, st)
    assert (b.S, b.G, b.N, b.E) == (1, 9, len(st["node_op"]), len(st["edge_src"]))
    v = b.host_view()
    gnp, gep = st["graph_node_ptr"], st["graph_edge_ptr"]
    eg = np.repeat(np.arange(b.G), np.diff(gep))               # graph of every input edge
    gsrc, gdst = st["edge_src"] + gnp[eg], st["edge_dst"] + gnp[eg]
    # receiver order: a stable sort of the input edges by global receiver
    order = np.argsort(gdst, kind="stable")
    assert np.array_equal(v["in_eid"], order)
    assert np.array_equal(v["in_dst"], gdst[order]) and np.array_equal(v["in_src"], gsrc[order])
    assert np.array_equal(v["edge_feat"], st["edge_feat"][order])
    assert np.array_equal(v["in_ptr"], np.concatenate([[0], np.cumsum(np.bincount(gdst, minlength=b.N))]))
    # sender-side index: positions grouped by sender, ascending
    assert np.array_equal(v["out_ptr"], np.concatenate([[0], np.cumsum(np.bincount(gsrc, minlength=b.N))]))
    assert sorted(v["out_pos"].tolist()) == list(range(b.E))
    for i in range(b.N):
        pos = v["out_pos"][v["out_ptr"][i]:v["out_ptr"][i + 1]]
        assert np.all(v["in_src"][pos] == i) and np.all(np.diff(pos) > 0)
    assert np.array_equal(v["node_graph"], np.repeat(np.arange(b.G), np.diff(gnp)))
    b.free()


def test_pack_edge_cases():
    m = base_model()
    # empty batch, zero-node graph, zero-edge graph, multi-edge and self-loop
    st = dict(n_states=0, state_graph_ptr=[0], graph_node_ptr=[0], graph_edge_ptr=[0], node_op=[],
              node_dense=np.zeros((0, 4)), edge_src=[], edge_dst=[], edge_feat=np.zeros((0, 8)),
              graph_global=None, slot_mask=[])
    b = xrl.pack_state(m, st)
    assert (b.S, b.G, b.N, b.E) == (0, 0, 0, 0)
    st = dict(n_states=1, state_graph_ptr=[0, 3], graph_node_ptr=[0, 0, 2, 5], graph_edge_ptr=[0, 0, 0, 4],
              node_op=[1, 2, 3, 4, 5], node_dense=np.ones((5, 4)), edge_src=[0, 0, 2, 1], edge_dst=[1, 1, 2, 0],
              edge_feat=np.arange(32).reshape(4, 8), graph_global=None, slot_mask=[1, 0, 1])
    v = xrl.pack_state(m, st).host_view()
    assert v["in_ptr"].tolist() == [0, 0, 0, 1, 3, 4]
    assert v["in_src"].tolist() == [3, 2, 2, 4] and v["in_eid"].tolist() == [3, 0, 1, 2]


def check_tiles(v):
    """Edge tiles: a partition of the receiver-order edges into runs of 1..32 edges whose
    boundaries fall between receivers, except inside a receiver with more than 32 in-edges; such a
    receiver starts a tile and is cut every 32 edges."""
    tp, in_ptr, in_dst = v["tile_ptr"], v["in_ptr"], v["in_dst"]
    E = len(in_dst)
    assert tp[0] == 0 and tp[-1] == E and (E > 0 or len(tp) == 1)
    sizes = np.diff(tp)
    assert np.all(sizes >= 1) and np.all(sizes <= 32)
    for t in tp[1:-1]:
        if in_dst[t - 1] == in_dst[t]:                       # the boundary cuts a receiver's range
            beg = in_ptr[in_dst[t]]
            assert in_ptr[in_dst[t] + 1] - beg > 32 and (t - beg) % 32 == 0
    # greedy: a tile is closed only when the next receiver's edges would not fit
    for i in range(len(tp) - 2):
        nxt = in_dst[tp[i + 1]]
        if in_dst[tp[i + 1] - 1] != nxt:
            deg = in_ptr[nxt + 1] - in_ptr[nxt]
            assert sizes[i] + min(deg, 32) > 32 or deg > 32


def test_edge_tiles():
    model, st = synth.make_config(1)
    check_tiles(xrl.pack_state(model, st).host_view())
    model, st = synth.make_config(2, n_cand=6)
    check_tiles(xrl.pack_state(model, st).host_view())
    rng = np.random.Generator(np.random.PCG64(5))
    for n_hub in (31, 32, 33, 64, 65, 300):                  # receivers of high in-degree
        n = n_hub + 40
        src = np.concatenate([np.arange(1, n_hub + 1), rng.integers(0, n, 60)]).astype(np.int32)
        dst = np.concatenate([np.full(n_hub, 7), rng.integers(0, n, 60)]).astype(np.int32)
        st = dict(n_states=1, state_graph_ptr=[0, 1], graph_node_ptr=[0, n], graph_edge_ptr=[0, len(src)],
                  node_op=np.zeros(n, np.int32), node_dense=np.zeros((n, 4)), edge_src=src, edge_dst=dst,
                  edge_feat=np.zeros((len(src), 8)), graph_global=None, slot_mask=[1])
        v = xrl.pack_state(base_model(), st).host_view()
        check_tiles(v)
        assert len(v["tile_ptr"]) - 1 >= -(-len(src) // 32)


def check_graph_tiles(v):
    """Per-graph edge tiles: every graph's in-edges partitioned into runs of 1..32 edges whose
    boundaries fall between receivers; no tile spans two graphs; greedy inside a graph."""
    gtp, tp, in_ptr, in_dst, gnp = v["graph_tile_ptr"], v["gtile_ptr"], v["in_ptr"], v["in_dst"], v["graph_node_ptr"]
    G, E = len(gnp) - 1, len(in_dst)
    assert len(gtp) == G + 1 and gtp[0] == 0 and gtp[-1] == len(tp) - 1 and tp[-1] == E
    for g in range(G):
        e0, e1 = in_ptr[gnp[g]], in_ptr[gnp[g + 1]]
        mine = tp[gtp[g]:gtp[g + 1] + 1]
        if e0 == e1:
            assert gtp[g] == gtp[g + 1]
            continue
        assert mine[0] == e0 and mine[-1] == e1
        sizes = np.diff(mine)
        assert np.all(sizes >= 1) and np.all(sizes <= 32)
        for i, t in enumerate(mine[1:-1]):
            assert in_dst[t - 1] != in_dst[t]
            deg = in_ptr[in_dst[t] + 1] - in_ptr[in_dst[t]]
            assert sizes[i] + deg > 32


def test_graph_edge_tiles():
    model, st = synth.make_config(1)
    check_graph_tiles(xrl.pack_state(model, st).host_view())
    model, st = synth.make_config(4, n_cand=5)
    check_graph_tiles(xrl.pack_state(model, st).host_view())
    # graphs without edges between graphs with edges, and at both ends
    n = 6
    st = dict(n_states=1, state_graph_ptr=[0, 5], graph_node_ptr=[0, n, 2 * n, 3 * n, 4 * n, 5 * n],
              graph_edge_ptr=[0, 0, 4, 4, 7, 7], node_op=np.zeros(5 * n, np.int32), node_dense=np.zeros((5 * n, 4)),
              edge_src=np.array([0, 1, 2, 3, 0, 1, 2], np.int32), edge_dst=np.array([1, 2, 3, 4, 5, 5, 3], np.int32),
              edge_feat=np.zeros((7, 8)), graph_global=None, slot_mask=[1] * 5)
    v = xrl.pack_state(base_model(), st).host_view()
    check_graph_tiles(v)
    assert list(v["graph_tile_ptr"]) == [0, 0, 1, 1, 2, 2]
    # a receiver of more than 32 in-edges: the batch has no per-graph tiles
    src = np.arange(1, 41).astype(np.int32)
    st = dict(n_states=1, state_graph_ptr=[0, 1], graph_node_ptr=[0, 50], graph_edge_ptr=[0, 40],
              node_op=np.zeros(50, np.int32), node_dense=np.zeros((50, 4)), edge_src=src,
              edge_dst=np.full(40, 7, np.int32), edge_feat=np.zeros((40, 8)), graph_global=None, slot_mask=[1])
    v = xrl.pack_state(base_model(), st).host_view()
    assert len(v["graph_tile_ptr"]) == 0 and len(v["gtile_ptr"]) == 0


def _mutate(st, **kw):
    out = {k: (np.array(v, copy=True) if isinstance(v, np.ndarray) else v) for k, v in st.items()}
    out.update(kw)
    return out


def test_pack_rejects_bad_input_with_error_codes():
    model, st = synth.make_config(1)
    E = xrl.ERR

    def code(state, m=model):
        with pytest.raises(xrl.XrlError) as ei:
            xrl.pack_state(m, state)
        assert len(str(ei.value)) > 20
        return ei.value.code

    bad = _mutate(st); bad["graph_node_ptr"][3] = bad["graph_node_ptr"][2] - 1
    assert code(bad) == E["SHAPE"]
    bad = _mutate(st); bad["state_graph_ptr"] = np.array([1, 9], np.int32)
    assert code(bad) == E["SHAPE"]
    assert code(_mutate(st, n_states=-1)) == E["SHAPE"]
    bad = _mutate(st, n_states=2, state_graph_ptr=np.array([0, 9, 9], np.int32))
    assert code(bad) == E["SHAPE"]                              # a state without its current graph
    bad = _mutate(st); bad["edge_dst"][5] = 10_000
    assert code(bad) == E["INDEX"]
    bad = _mutate(st); bad["edge_src"][0] = -1
    assert code(bad) == E["INDEX"]
    bad = _mutate(st); bad["node_op"][7] = 32
    assert code(bad) == E["INDEX"]
    bad = _mutate(st); bad["edge_feat"][3, 2] = np.nan
    assert code(bad) == E["VALUE"]
    bad = _mutate(st); bad["node_dense"][0, 0] = np.inf
    assert code(bad) == E["VALUE"]
    bad = _mutate(st); bad["slot_mask"][0] = 0
    assert code(bad) == E["MASK"]
    assert code(_mutate(st, node_op=None)) == E["NULL"]
    assert code(st, base_model(hidden=0)) == E["SHAPE"]
    assert code(st, base_model(readout=7)) == E["SHAPE"]
    lib = xrl.load_library()
    assert lib.xrl_pack_state(None, None, None) == E["NULL"]
    assert lib.xrl_weight_count(None) == E["NULL"]
    assert lib.xrl_batch_free(None) == 0 and lib.xrl_destroy(None) == 0


def test_device_calls_fail_cleanly_without_gpu_or_upload():
    import torch
    lib = xrl.load_library()
    model, st = synth.make_config(1)
    assert lib.xrl_create(None, None, None, None) == xrl.ERR["NULL"]
    w = np.zeros(xrl.weight_count(model), np.float32)
    h = C.c_void_p()
    for kw in (dict(hidden=96), dict(mlp_layers=3)):
        md = xrl.model_desc(base_model(**kw))
        w2 = np.zeros(xrl.weight_count(base_model(**kw)), np.float32)
        assert lib.xrl_create(C.byref(md), w2.ctypes.data, None, C.byref(h)) == xrl.ERR["UNSUPPORTED"]
    if not torch.cuda.is_available():
        md = xrl.model_desc(model)
        assert lib.xrl_create(C.byref(md), w.ctypes.data, None, C.byref(h)) == xrl.ERR["HIP"]
        with pytest.raises(RuntimeError):
            xrl.Encoder(model, w)
    b = xrl.pack_state(model, st)
    assert lib.xrl_encode(None, b.handle, None, 0) == xrl.ERR["NULL"]


def test_shape_features_host_call():
    """xrl_edge_features_from_shapes against the oracle's (random shapes of rank 0..4) and the
    paper's printed example; error codes for bad input."""
    import ctypes as C
    from oracle import xrl_oracle as O
    rng = np.random.default_rng(9)
    shapes = [[1, 3, 256, 256]] + [list(rng.integers(0, 5000, size=int(rng.integers(0, 5)))) for _ in range(200)]
    got = xrl.edge_features_from_shapes(shapes)
    ref = O.edge_features_from_shapes(shapes)
    assert got.dtype == np.float32 and got.shape == (201, 4)
    np.testing.assert_array_equal(got, ref.astype(np.float32))
    np.testing.assert_array_equal(got[0], np.float32([1 / 4096, 3 / 4096, 0.0625, 0.0625]))
    assert xrl.edge_features_from_shapes([]).shape == (0, 4)
    for bad, code in (([[1, 2, 3, 4, 5]], "SHAPE"), ([[3, -1]], "VALUE")):
        with pytest.raises(xrl.XrlError) as ei:
            xrl.edge_features_from_shapes(bad)
        assert ei.value.code == xrl.ERR[code]
    with pytest.raises(xrl.XrlError) as ei:
        xrl.edge_features_from_shapes([[1]], M=0.0)
    assert ei.value.code == xrl.ERR["VALUE"]


def test_threaded_pack_equals_serial(monkeypatch):
    """The packer cuts large batches into graph ranges, one per thread (XRL_PACK_THREADS forces the
    count): every packed array must be identical to the serial result, for thread counts below,
    at and above the number of graphs, and errors must be reported as a serial pass finds them."""
    model, st = synth.make_config(3, n_states=2)
    monkeypatch.setenv("XRL_PACK_THREADS", "1")
    b = xrl.pack_state(model, st)
    ref = b.host_view()
    check_tiles(ref)
    b.free()
    G = len(st["graph_node_ptr"]) - 1
    for t in (2, 7, G, G + 5):
        monkeypatch.setenv("XRL_PACK_THREADS", str(t))
        b = xrl.pack_state(model, st)
        v = b.host_view()
        b.free()
        for k in ref:
            np.testing.assert_array_equal(v[k], ref[k], err_msg=f"{k} with {t} threads")
    # a bad operator id late in the batch and a bad edge early: the operator id is reported
    # (operator ids are checked before edges), whatever the thread count
    bad = _mutate(st)
    bad["node_op"][-3] = 999
    bad["edge_dst"][2] = 10_000_000
    for t in ("1", "7"):
        monkeypatch.setenv("XRL_PACK_THREADS", t)
        with pytest.raises(xrl.XrlError) as ei:
            xrl.pack_state(model, bad)
        assert ei.value.code == xrl.ERR["INDEX"] and "op id 999" in str(ei.value)
    # two bad edges: the one with the lower index is reported
    bad = _mutate(st)
    bad["edge_src"][5] = -7
    bad["edge_src"][len(bad["edge_src"]) - 1] = -9
    monkeypatch.setenv("XRL_PACK_THREADS", "7")
    with pytest.raises(xrl.XrlError) as ei:
        xrl.pack_state(model, bad)
    assert "(-7 ->" in str(ei.value)


def test_public_header_is_plain_c(tmp_path):
    """include/xrl.h is the boundary: it must compile as C99 on its own (no C++, no HIP or torch types)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "h.c"
    src.write_text('#include "xrl.h"\nint main(void) { return XRL_OK; }\n')
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
