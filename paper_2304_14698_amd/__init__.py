"""Python binding of libxrl (see include/xrl.h): argument marshalling only.

Every step of the path runs inside the HIP library; torch is used for device buffers and the
stream handle. There is no CPU fallback: if the library is missing, load_library() raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("XRL_LIBRARY") or os.path.join(_HERE, "libxrl.so")
_lib = None

PRECISION = {"fp32": 0, "bf16": 1}
READOUT = {"sum": 0, "mean": 1}
ROUND_KIND = {"mlp": 0, "gat": 1}


class XrlError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"xrl error {code}: {msg}")
        self.code = code


ERR = dict(NULL=-1, SHAPE=-2, INDEX=-3, VALUE=-4, MASK=-5, STATE=-6, UNSUPPORTED=-7, OOM=-8, HIP=-9)


class ModelDesc(C.Structure):
    _fields_ = [("n_op_types", C.c_int32), ("n_node_dense", C.c_int32), ("d_edge", C.c_int32),
                ("d_global", C.c_int32), ("hidden", C.c_int32), ("rounds", C.c_int32),
                ("mlp_layers", C.c_int32), ("head_hidden", C.c_int32 * 2),
                ("readout", C.c_int32), ("precision", C.c_int32), ("round_kind", C.c_int32)]


class StateDesc(C.Structure):
    _fields_ = [("n_states", C.c_int32),
                ("state_graph_ptr", C.c_void_p), ("graph_node_ptr", C.c_void_p),
                ("graph_edge_ptr", C.c_void_p), ("node_op", C.c_void_p),
                ("node_dense", C.c_void_p), ("edge_src", C.c_void_p), ("edge_dst", C.c_void_p),
                ("edge_feat", C.c_void_p), ("graph_global", C.c_void_p), ("slot_mask", C.c_void_p)]


class EditStateDesc(C.Structure):
    _fields_ = [("n_states", C.c_int32)] + [(k, C.c_void_p) for k in (
        "cur_node_ptr", "cur_edge_ptr", "node_op", "node_dense", "edge_src", "edge_dst", "edge_feat",
        "state_cand_ptr", "del_node_ptr", "del_node", "del_edge_ptr", "del_edge", "add_node_ptr",
        "add_node_op", "add_node_dense", "add_edge_ptr", "add_edge_src", "add_edge_dst", "add_edge_feat",
        "graph_global", "slot_mask")]


class PackedView(C.Structure):
    _fields_ = [("S", C.c_int64), ("G", C.c_int64), ("N", C.c_int64), ("E", C.c_int64),
                ("state_graph_ptr", C.c_void_p), ("graph_node_ptr", C.c_void_p),
                ("in_ptr", C.c_void_p), ("in_src", C.c_void_p), ("in_dst", C.c_void_p),
                ("in_eid", C.c_void_p), ("out_ptr", C.c_void_p), ("out_pos", C.c_void_p),
                ("node_graph", C.c_void_p), ("edge_feat", C.c_void_p),
                ("n_tiles", C.c_int64), ("tile_ptr", C.c_void_p),
                ("n_graph_tiles", C.c_int64), ("graph_tile_ptr", C.c_void_p), ("gtile_ptr", C.c_void_p)]


EXPORTS = ["xrl_weight_count", "xrl_weight_tensor_count", "xrl_weight_tensor", "xrl_pack_state", "xrl_pack_state_edits",
           "xrl_batch_dims", "xrl_batch_host_view", "xrl_batch_free", "xrl_create",
           "xrl_set_weights", "xrl_destroy", "xrl_batch_upload", "xrl_encode", "xrl_policy_value",
           "xrl_policy_value_static",
           "xrl_policy_value_backward", "xrl_encode_backward", "xrl_ppo_objective", "xrl_segment_sum",
           "xrl_get_activation", "xrl_set_timing", "xrl_read_timing", "xrl_measure_peaks",
           "xrl_edge_features_from_shapes", "xrl_weight_gradient", "xrl_mlp_backward", "xrl_last_error", "xrl_version"]


def load_library():
    """Loads libxrl.so (built by __graft_entry__.build()); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise OSError(f"{LIB_PATH} not found: run `python __graft_entry__.py` to build it")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.xrl_weight_count.restype = i64
    lib.xrl_weight_count.argtypes = [C.POINTER(ModelDesc)]
    lib.xrl_weight_tensor_count.restype = i32
    lib.xrl_weight_tensor_count.argtypes = [C.POINTER(ModelDesc)]
    lib.xrl_weight_tensor.argtypes = [C.POINTER(ModelDesc), i32, C.c_char_p, C.c_size_t,
                                      C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    lib.xrl_pack_state.argtypes = [C.POINTER(ModelDesc), C.POINTER(StateDesc), C.POINTER(vp)]
    lib.xrl_pack_state_edits.argtypes = [C.POINTER(ModelDesc), C.POINTER(EditStateDesc), C.POINTER(vp)]
    lib.xrl_batch_dims.argtypes = [vp] + [C.POINTER(i64)] * 4
    lib.xrl_batch_host_view.argtypes = [vp, C.POINTER(PackedView)]
    lib.xrl_batch_free.argtypes = [vp]
    lib.xrl_create.argtypes = [C.POINTER(ModelDesc), vp, vp, C.POINTER(vp)]
    lib.xrl_set_weights.argtypes = [vp, vp]
    lib.xrl_destroy.argtypes = [vp]
    lib.xrl_batch_upload.argtypes = [vp, vp]
    lib.xrl_encode.argtypes = [vp, vp, vp, C.c_int]
    lib.xrl_policy_value.argtypes = [vp] * 8
    lib.xrl_policy_value_static.argtypes = [vp] * 8
    lib.xrl_policy_value_backward.argtypes = [vp] * 8
    lib.xrl_encode_backward.argtypes = [vp] * 4
    lib.xrl_segment_sum.argtypes = [vp, vp, vp, i64, i64, i32, vp]
    lib.xrl_edge_features_from_shapes.argtypes = [vp, vp, i64, C.c_double, vp]
    lib.xrl_weight_gradient.argtypes = [vp, vp, i32, vp, vp, vp, i64, vp, vp]
    lib.xrl_mlp_backward.argtypes = [vp, vp, i32, i32] + [vp] * 9
    lib.xrl_get_activation.argtypes = [vp, vp, C.c_char_p, i32, vp]
    lib.xrl_set_timing.argtypes = [vp, C.c_int]
    lib.xrl_read_timing.argtypes = [vp, C.c_char_p, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.xrl_measure_peaks.argtypes = [vp, i64, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.xrl_ppo_objective.argtypes = [vp] * 9 + [C.c_float] * 3 + [vp] * 4
    lib.xrl_last_error.restype = C.c_char_p
    lib.xrl_version.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc):
    if rc < 0:
        raise XrlError(int(rc), load_library().xrl_last_error().decode())
    return rc


def model_desc(model):
    hh = model.get("head_hidden", (256, 64))
    prec, ro = model.get("precision", "fp32"), model.get("readout", "sum")
    return ModelDesc(model["n_op_types"], model["n_node_dense"], model["d_edge"], model["d_global"],
                     model["hidden"], model["rounds"], model.get("mlp_layers", 2),
                     (C.c_int32 * 2)(int(hh[0]), int(hh[1])),
                     READOUT[ro] if isinstance(ro, str) else int(ro),
                     PRECISION[prec] if isinstance(prec, str) else int(prec),
                     ROUND_KIND[model.get("round_kind", "mlp")])


def weight_count(model):
    return _check(load_library().xrl_weight_count(C.byref(model_desc(model))))


def weight_layout(model):
    """[(name, shape)] in flat-vector order, as the library lays the weights out."""
    lib, md = load_library(), model_desc(model)
    n = _check(lib.xrl_weight_tensor_count(C.byref(md)))
    out, expect = [], 0
    for i in range(n):
        name = C.create_string_buffer(64)
        off, rows, cols = C.c_int64(), C.c_int64(), C.c_int64()
        _check(lib.xrl_weight_tensor(C.byref(md), i, name, 64, C.byref(off), C.byref(rows), C.byref(cols)))
        assert off.value == expect
        shape = (rows.value, cols.value) if cols.value else (rows.value,)
        expect += int(np.prod(shape))
        out.append((name.value.decode(), shape))
    return out


def _arr(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _ptr(a):
    return None if a is None else a.ctypes.data


class Batch:
    """A packed meta-batch (host side; device side after Encoder.upload)."""

    def __init__(self, model, state, edits=False):
        lib = load_library()
        self.handle = C.c_void_p()
        self.model = dict(model)
        if edits:
            # candidates given as edits of each state's current graph (see xrl_edit_state_desc)
            f32 = ("node_dense", "edge_feat", "add_node_dense", "add_edge_feat", "graph_global")
            keep = {k: _arr(state.get(k), np.float32 if k in f32 else (np.uint8 if k == "slot_mask" else np.int32))
                    for k, _ in EditStateDesc._fields_[1:]}
            sd = EditStateDesc(int(state["n_states"]), *[_ptr(keep[k]) for k, _ in EditStateDesc._fields_[1:]])
            _check(lib.xrl_pack_state_edits(C.byref(model_desc(model)), C.byref(sd), C.byref(self.handle)))
            d = [C.c_int64() for _ in range(4)]
            _check(lib.xrl_batch_dims(self.handle, *[C.byref(x) for x in d]))
            self.S, self.G, self.N, self.E = (int(x.value) for x in d)
            return
        self._keep = dict(
            sgp=_arr(state["state_graph_ptr"], np.int32), gnp=_arr(state["graph_node_ptr"], np.int32),
            gep=_arr(state["graph_edge_ptr"], np.int32), op=_arr(state["node_op"], np.int32),
            dense=_arr(state.get("node_dense"), np.float32), src=_arr(state["edge_src"], np.int32),
            dst=_arr(state["edge_dst"], np.int32), ef=_arr(state["edge_feat"], np.float32),
            gg=_arr(state.get("graph_global"), np.float32), mask=_arr(state["slot_mask"], np.uint8))
        k = self._keep
        sd = StateDesc(int(state["n_states"]), _ptr(k["sgp"]), _ptr(k["gnp"]), _ptr(k["gep"]),
                       _ptr(k["op"]), _ptr(k["dense"]), _ptr(k["src"]), _ptr(k["dst"]),
                       _ptr(k["ef"]), _ptr(k["gg"]), _ptr(k["mask"]))
        _check(lib.xrl_pack_state(C.byref(model_desc(model)), C.byref(sd), C.byref(self.handle)))
        self._keep = None                      # host inputs are only borrowed during the call
        d = [C.c_int64() for _ in range(4)]
        _check(lib.xrl_batch_dims(self.handle, *[C.byref(x) for x in d]))
        self.S, self.G, self.N, self.E = (int(x.value) for x in d)

    def host_view(self):
        """Copies of the packed host arrays as numpy arrays."""
        v = PackedView()
        _check(load_library().xrl_batch_host_view(self.handle, C.byref(v)))
        De = self.model["d_edge"]

        def grab(p, n, ct=C.c_int32, dt=np.int32):
            if n == 0:
                return np.zeros(0, dtype=dt)
            return np.ctypeslib.as_array(C.cast(p, C.POINTER(ct)), shape=(n,)).astype(dt, copy=True)
        return dict(state_graph_ptr=grab(v.state_graph_ptr, self.S + 1),
                    graph_node_ptr=grab(v.graph_node_ptr, self.G + 1),
                    in_ptr=grab(v.in_ptr, self.N + 1), in_src=grab(v.in_src, self.E),
                    in_dst=grab(v.in_dst, self.E), in_eid=grab(v.in_eid, self.E),
                    out_ptr=grab(v.out_ptr, self.N + 1), out_pos=grab(v.out_pos, self.E),
                    node_graph=grab(v.node_graph, self.N),
                    tile_ptr=grab(v.tile_ptr, int(v.n_tiles) + 1),
                    graph_tile_ptr=grab(v.graph_tile_ptr, self.G + 1 if v.graph_tile_ptr else 0),
                    gtile_ptr=grab(v.gtile_ptr, int(v.n_graph_tiles) + 1 if v.gtile_ptr else 0),
                    edge_feat=grab(v.edge_feat, self.E * De, C.c_float, np.float32).reshape(self.E, De))

    def free(self):
        if self.handle:
            load_library().xrl_batch_free(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def pack_state(model, state):
    return Batch(model, state)


def pack_state_edits(model, edit_state):
    """Packs states whose candidates are edits of the current graph (xrl_pack_state_edits)."""
    return Batch(model, edit_state, edits=True)


def edge_features_from_shapes(shapes, M=4096.0):
    """[E, 4] float32 edge attributes from a list of tensor shapes (rank <= 4 each)."""
    lib = load_library()
    ptr = np.zeros(len(shapes) + 1, dtype=np.int32)
    ptr[1:] = np.cumsum([len(sh) for sh in shapes])
    dims = np.ascontiguousarray([d for sh in shapes for d in sh], dtype=np.int64)
    out = np.empty((len(shapes), 4), dtype=np.float32)
    _check(lib.xrl_edge_features_from_shapes(ptr.ctypes.data, dims.ctypes.data if dims.size else None,
                                             len(shapes), C.c_double(M), out.ctypes.data))
    return out


class Encoder:
    """Device context: weights + workspaces on the current torch CUDA stream."""

    def __init__(self, model, weights, stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("xrl needs a GPU: torch.cuda.is_available() is False")
        self.torch = torch
        self.model = dict(model)
        self.lib = load_library()
        self.H = model["hidden"]
        self.n_weights = weight_count(model)
        w = np.ascontiguousarray(weights, dtype=np.float32)
        if w.size != self.n_weights:
            raise ValueError(f"weights has {w.size} entries, the model needs {self.n_weights}")
        self.stream = torch.cuda.current_stream() if stream is None else stream
        self.handle = C.c_void_p()
        _check(self.lib.xrl_create(C.byref(model_desc(model)), w.ctypes.data,
                                   C.c_void_p(self.stream.cuda_stream), C.byref(self.handle)))

    def set_weights(self, weights):
        w = np.ascontiguousarray(weights, dtype=np.float32)
        assert w.size == self.n_weights
        _check(self.lib.xrl_set_weights(self.handle, w.ctypes.data))

    def upload(self, batch):
        _check(self.lib.xrl_batch_upload(self.handle, batch.handle))
        return batch

    def pack(self, state):
        return self.upload(Batch(self.model, state))

    def pack_edits(self, edit_state):
        return self.upload(Batch(self.model, edit_state, edits=True))

    def _empty(self, shape, dtype=None):
        t = self.torch
        return t.empty(shape, dtype=dtype or t.float32, device="cuda")

    def encode(self, batch, save_for_backward=False, out=None):
        emb = self._empty((batch.G, self.H)) if out is None else out
        _check(self.lib.xrl_encode(self.handle, batch.handle, emb.data_ptr(), int(save_for_backward)))
        return emb

    def policy_value(self, batch, emb, out=None, static=False):
        """static=True: the entry point that allocates nothing (`out` must then be given)."""
        t = self.torch
        o = out or dict(logp=self._empty((batch.G,)), value=self._empty((batch.S,)),
                        entropy=self._empty((batch.S,)), action=self._empty((batch.S,), t.int32),
                        logit=self._empty((batch.G,)))
        fn = self.lib.xrl_policy_value_static if static else self.lib.xrl_policy_value
        logit = o.get("logit")
        _check(fn(self.handle, batch.handle, emb.data_ptr(), o["logp"].data_ptr(),
                  o["value"].data_ptr(), o["entropy"].data_ptr(),
                  o["action"].data_ptr(), None if logit is None else logit.data_ptr()))
        return o

    def policy_value_backward(self, batch, emb, dlogp, dvalue, dentropy, dweights):
        demb = self._empty((batch.G, self.H))
        _check(self.lib.xrl_policy_value_backward(self.handle, batch.handle, emb.data_ptr(),
                                                  dlogp.data_ptr(), dvalue.data_ptr(),
                                                  dentropy.data_ptr(), demb.data_ptr(),
                                                  dweights.data_ptr()))
        return demb

    def ppo_objective(self, batch, pv, action, old_logp, advantage, v_target, eps=0.2, c1=0.5, c2=0.01):
        """(J [4] = J, L_clip, L_vf, L_entropy; dlogp [G]; dvalue [S]; dentropy [S]) from the outputs
        `pv` of policy_value and the rollout's records (device tensors)."""
        J, dlogp = self._empty((4,)), self._empty((batch.G,))
        dvalue, dentropy = self._empty((batch.S,)), self._empty((batch.S,))
        _check(self.lib.xrl_ppo_objective(self.handle, batch.handle, pv["logp"].data_ptr(), pv["value"].data_ptr(),
                                          pv["entropy"].data_ptr(), action.data_ptr(), old_logp.data_ptr(),
                                          advantage.data_ptr(), v_target.data_ptr(), eps, c1, c2, J.data_ptr(),
                                          dlogp.data_ptr(), dvalue.data_ptr(), dentropy.data_ptr()))
        return J, dlogp, dvalue, dentropy

    def encode_backward(self, batch, demb, dweights):
        _check(self.lib.xrl_encode_backward(self.handle, batch.handle, demb.data_ptr(), dweights.data_ptr()))
        return dweights

    def mlp_backward(self, batch, kind, rnd, h, dy, agg=None, y=None):
        """Gradients through the edge / node MLP of round `rnd` on given inputs (see xrl.h):
        returns dict(z1, dz1, dz2, dxa, dxb), tensors of the operand type."""
        t = self.torch
        rows = batch.E if kind == "edge" else batch.N
        o = {k: t.empty((rows, self.H), dtype=h.dtype, device="cuda") for k in ("z1", "dz1", "dz2", "dxa", "dxb")}
        p = lambda x: None if x is None else x.data_ptr()
        _check(self.lib.xrl_mlp_backward(self.handle, batch.handle, dict(edge=1, node=2)[kind], rnd, p(h), p(agg),
                                         p(y), p(dy), p(o["z1"]), p(o["dz1"]), p(o["dz2"]), p(o["dxa"]), p(o["dxb"])))
        return o

    def weight_gradient(self, batch, kind, x, dz, dW, db, x2=None):
        """dW += X^T dz, db += column sums of dz (kind: "plain" | "edge" | "node"; see xrl.h)."""
        k = dict(plain=0, edge=1, node=2)[kind]
        _check(self.lib.xrl_weight_gradient(self.handle, batch.handle, k, x.data_ptr(),
                                            x2.data_ptr() if x2 is not None else None, dz.data_ptr(),
                                            x.shape[0], dW.data_ptr(), db.data_ptr()))
        return dW, db

    def segment_sum(self, values, ptr, out=None):
        n_rows, width = values.shape
        n_seg = ptr.numel() - 1
        o = self._empty((n_seg, width)) if out is None else out
        _check(self.lib.xrl_segment_sum(self.handle, values.data_ptr(), ptr.data_ptr(), n_rows, n_seg,
                                        width, o.data_ptr()))
        return o

    def get_activation(self, batch, what, rnd=0):
        shape = {"a0": (batch.N, self.model["d_edge"]), "pool": (batch.G, self.H)}.get(what, (batch.N, self.H))
        o = self._empty(shape)
        _check(self.lib.xrl_get_activation(self.handle, batch.handle, what.encode(), rnd, o.data_ptr()))
        return o

    def set_timing(self, enabled):
        _check(self.lib.xrl_set_timing(self.handle, int(enabled)))

    def read_timing(self, kernel):
        """(total milliseconds, launches) recorded for `kernel` since the last read."""
        ms, n = C.c_double(), C.c_int64()
        _check(self.lib.xrl_read_timing(self.handle, kernel.encode(), C.byref(ms), C.byref(n)))
        return ms.value, int(n.value)

    def measure_peaks(self, copy_bytes=1 << 30):
        """(bf16 MFMA TFLOP/s of a register-resident loop, GB/s of a device-to-device copy)."""
        tf, gb = C.c_double(), C.c_double()
        _check(self.lib.xrl_measure_peaks(self.handle, int(copy_bytes), C.byref(tf), C.byref(gb)))
        return tf.value, gb.value

    def close(self):
        if self.handle:
            self.lib.xrl_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
