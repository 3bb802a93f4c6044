"""Float64 CPU oracle of the graph-rewrite agent's state encoder, policy head and value head.

TEST INFRASTRUCTURE ONLY. This module is the slow, literal definition that the GPU library is
checked against; nothing in the product path may import it, and it imports nothing from the
product. It works on the unsorted edge list, one graph at a time, in numpy float64.

What it follows (X-RLflow, arXiv 2304.14698):
  * Section 3.4, node-update layer (first equation of 3.4): every node sums the attributes of
    its incoming edges, concatenates its own attribute, and applies a learned layer + sigma.
  * Section 3.4, k message-passing layers (second equation of 3.4): a learned per-edge
    function of the sender state is summed at the receiver, followed by sigma. Two readings
    are implemented: round_kind="mlp" (edge-MLP on [h_src | h_dst | e], sum at the receiver,
    node-MLP on [h | sum]) and round_kind="gat" (the cited graph-attention layer: z = hW,
    logits LeakyReLU_0.2(a_s.z_src + a_d.z_dst), softmax over a receiver's in-edges plus a
    self edge, h' = ReLU(sum alpha z)).
  * Section 3.4, global-update layer (third equation of 3.4): all node states of a graph are
    summed (or averaged), concatenated with the graph's global attribute (zero by default,
    Section 3.3.2) and passed through a learned layer + sigma.
  * Section 3.3.2: the per-graph representations of a state (current graph = No-Op slot 0,
    then the candidates) feed a policy head (categorical over valid slots; invalid slots are
    masked out exactly) and a value head; both heads are MLPs with hidden sizes [256, 64]
    (hyper-parameter table in the appendix).
  * Section 3.3.4: everything is trained by one back-propagation; the backward functions here
    are hand-written reverse-mode code, separate from the forward functions. ppo_objective is
    the section's objective J = L_clip + c1 L_vf + c2 L_entropy (its three equations; c1 = 0.5,
    c2 = 0.01 in the appendix table) with its derivatives w.r.t. the heads' outputs.

Conventions: row vectors, y = x W + b with W stored [in, out]; sigma = ReLU after every encoder
layer (including each MLP's last), heads end with a linear layer of width 1.

Pinned by tests/test_oracle_pins.py (dense-adjacency brute force, a hand-worked example,
relabelling and batch invariance, softmax identities, adjoint identities, finite differences).
Parity unpinned: which action a *trained* agent would choose (needs the paper's weights).
"""
import numpy as np

F = np.float64


def default_model(**kw):
    m = dict(n_op_types=32, n_node_dense=4, d_edge=8, d_global=1, hidden=64, rounds=2,
             mlp_layers=2, head_hidden=(256, 64), readout="sum", round_kind="mlp")
    m.update(kw)
    return m


# ----------------------------------------------------------------------------- weights
def _mlp_shapes(prefix, d_in, widths):
    out, d = [], d_in
    for i, w in enumerate(widths):
        out.append((f"{prefix}.W{i}", (d, w)))
        out.append((f"{prefix}.b{i}", (w,)))
        d = w
    return out


def weight_layout(model):
    """Order of tensors in the flat weight vector: embed MLP, then per round (edge MLP, node
    MLP) or (GAT W, a_src, a_dst), readout MLP, policy head, value head."""
    H, L = model["hidden"], model["mlp_layers"]
    De, Dn = model["d_edge"], model["n_op_types"] + model["n_node_dense"]
    lay = _mlp_shapes("embed", De + Dn, [H] * L)
    for r in range(model["rounds"]):
        if model.get("round_kind", "mlp") == "gat":
            lay += [(f"gat{r}.W", (H, H)), (f"gat{r}.a_src", (H,)), (f"gat{r}.a_dst", (H,))]
        else:
            lay += _mlp_shapes(f"edge{r}", 2 * H + De, [H] * L)
            lay += _mlp_shapes(f"node{r}", 2 * H, [H] * L)
    lay += _mlp_shapes("readout", H + model["d_global"], [H] * L)
    hh = list(model["head_hidden"])
    lay += _mlp_shapes("policy", H, hh + [1])
    lay += _mlp_shapes("value", H, hh + [1])
    return lay


def weight_count(model):
    return int(sum(int(np.prod(s)) for _, s in weight_layout(model)))


def unflatten(model, w):
    w = np.asarray(w, dtype=F).ravel()
    out, o = {}, 0
    for name, shape in weight_layout(model):
        n = int(np.prod(shape))
        out[name] = w[o:o + n].reshape(shape)
        o += n
    if o != w.size:
        raise ValueError(f"weight vector has {w.size} entries, layout needs {o}")
    return out


def flatten(model, d):
    return np.concatenate([np.asarray(d[name], dtype=F).ravel() for name, _ in weight_layout(model)])


def _layers(W, prefix):
    out, i = [], 0
    while f"{prefix}.W{i}" in W:
        out.append((W[f"{prefix}.W{i}"], W[f"{prefix}.b{i}"]))
        i += 1
    return out


# ----------------------------------------------------------------------------- MLP
def mlp_forward(x, layers, last_relu):
    """Returns the output and, per layer, (input, pre-activation)."""
    cache = []
    for i, (Wm, b) in enumerate(layers):
        z = x @ Wm + b
        cache.append((x, z))
        x = np.maximum(z, 0.0) if (last_relu or i + 1 < len(layers)) else z
    return x, cache


def mlp_backward(dy, layers, cache, last_relu, bound=None):
    """Reverse of mlp_forward: returns dx and [(dW, db)] in layer order. If `bound` is a list,
    it receives per layer (|x|^T |dz|, sum |dz|): the sums of absolute terms of each gradient
    entry, i.e. the quantity a rounding-error bound of that entry is proportional to."""
    grads = [None] * len(layers)
    for i in reversed(range(len(layers))):
        Wm, _ = layers[i]
        x, z = cache[i]
        dz = dy * (z > 0.0) if (last_relu or i + 1 < len(layers)) else dy
        grads[i] = (x.T @ dz, dz.sum(axis=0))
        if bound is not None:
            bound.insert(0, (np.abs(x).T @ np.abs(dz), np.abs(dz).sum(axis=0)))
        dy = dz @ Wm.T
    return dy, grads


# ----------------------------------------------------------------------------- graph access
def graph_slices(state, g):
    n0, n1 = int(state["graph_node_ptr"][g]), int(state["graph_node_ptr"][g + 1])
    e0, e1 = int(state["graph_edge_ptr"][g]), int(state["graph_edge_ptr"][g + 1])
    return slice(n0, n1), slice(e0, e1)


def node_features(model, op, dense):
    """x_i = [onehot(op_i) | dense_i] (Section 3.3.2: one-hot of the operator index)."""
    n, T = op.shape[0], model["n_op_types"]
    x = np.zeros((n, T + model["n_node_dense"]), dtype=F)
    x[np.arange(n), op] = 1.0
    x[:, T:] = dense
    return x


def edge_features_from_shapes(shapes, M=4096.0):
    """Section 3.3.2, paragraph on the graph input: an edge's attribute is its tensor's shape,
    zero-padded on the leading side to rank 4, divided by the constant M of the appendix's
    hyper-parameter table (4096)."""
    out = np.zeros((len(shapes), 4), dtype=F)
    for e, sh in enumerate(shapes):
        sh = list(sh)
        assert len(sh) <= 4 and all(d >= 0 for d in sh)
        for k, d in enumerate(sh):
            out[e, 4 - len(sh) + k] = d / M
    return out


def segment_sum(values, index, n):
    """out[i] = sum of values[e] over e with index[e] == i."""
    out = np.zeros((n,) + values.shape[1:], dtype=F)
    np.add.at(out, index, values)
    return out


def _leaky(x, slope=0.2):
    return np.where(x > 0.0, x, slope * x)


# ----------------------------------------------------------------------------- encoder forward
def encode_graph(model, W, op, dense, src, dst, xe, gglob):
    """One graph -> dict with every intermediate; 'emb' is the graph representation u_g."""
    n, H = op.shape[0], model["hidden"]
    xe = np.asarray(xe, dtype=F).reshape(src.shape[0], model["d_edge"])
    x = node_features(model, op, np.asarray(dense, dtype=F).reshape(n, model["n_node_dense"]))
    a0 = segment_sum(xe, dst, n)                                   # node-update layer
    h, c_embed = mlp_forward(np.concatenate([a0, x], axis=1), _layers(W, "embed"), True)
    out = dict(a0=a0, h=[h], agg=[], c_embed=c_embed, c_edge=[], c_node=[], gat=[])
    for r in range(model["rounds"]):
        if model.get("round_kind", "mlp") == "gat":
            Wg, a_s, a_d = W[f"gat{r}.W"], W[f"gat{r}.a_src"], W[f"gat{r}.a_dst"]
            z = h @ Wg
            s_edge = _leaky(z[src] @ a_s + z[dst] @ a_d)
            s_self = _leaky(z @ a_s + z @ a_d)
            mx = s_self.copy()
            np.maximum.at(mx, dst, s_edge)
            w_edge, w_self = np.exp(s_edge - mx[dst]), np.exp(s_self - mx)
            den = w_self + segment_sum(w_edge, dst, n)
            alpha_e, alpha_s = w_edge / den[dst], w_self / den
            pre = segment_sum(alpha_e[:, None] * z[src], dst, n) + alpha_s[:, None] * z
            out["gat"].append(dict(z=z, alpha_e=alpha_e, alpha_s=alpha_s, pre=pre))
            h = np.maximum(pre, 0.0)
        else:
            xin = np.concatenate([h[src], h[dst], xe], axis=1)
            m, c_e = mlp_forward(xin, _layers(W, f"edge{r}"), True)
            agg = segment_sum(m, dst, n)
            h, c_n = mlp_forward(np.concatenate([h, agg], axis=1), _layers(W, f"node{r}"), True)
            out["agg"].append(agg); out["c_edge"].append(c_e); out["c_node"].append(c_n)
        out["h"].append(h)
    pool = h.sum(axis=0) if n > 0 else np.zeros(H, dtype=F)        # global-update layer
    if model["readout"] == "mean":
        pool = pool / max(n, 1)
    gin = np.concatenate([pool, np.asarray(gglob, dtype=F).ravel()])[None, :]
    u, c_g = mlp_forward(gin, _layers(W, "readout"), True)
    out.update(pool=pool, c_readout=c_g, emb=u[0])
    return out


def _graph_args(state, g):
    ns, es = graph_slices(state, g)
    gg = state.get("graph_global")
    return (state["node_op"][ns], state["node_dense"][ns], state["edge_src"][es],
            state["edge_dst"][es], state["edge_feat"][es],
            gg[g] if gg is not None else None)


def encode(model, w, state, keep=False, graphs=None):
    """Embeddings [G, H] of every graph (slot) of the meta-batch. keep=True also returns the
    list of per-graph intermediate dicts. `graphs` restricts to a subset of graph indices."""
    W = unflatten(model, w)
    G = len(state["graph_node_ptr"]) - 1
    idx = range(G) if graphs is None else graphs
    emb, inter = np.zeros((len(idx), model["hidden"]), dtype=F), []
    for k, g in enumerate(idx):
        op, dense, src, dst, xe, gg = _graph_args(state, g)
        if gg is None:
            gg = np.zeros(model["d_global"])
        o = encode_graph(model, W, op, dense, src, dst, xe, gg)
        emb[k] = o["emb"]
        if keep:
            inter.append(o)
    return (emb, inter) if keep else emb


# ----------------------------------------------------------------------------- heads forward
def policy_value(model, w, emb, state):
    """Per slot: logit, logp (-inf when masked), p (0 when masked). Per state: entropy, action
    (slot index inside the state, 0 = No-Op, lowest index among maxima), value."""
    W = unflatten(model, w)
    emb = np.asarray(emb, dtype=F)
    sgp, mask = state["state_graph_ptr"], np.asarray(state["slot_mask"]).astype(bool)
    S, G = len(sgp) - 1, emb.shape[0]
    logit, c_pi = mlp_forward(emb, _layers(W, "policy"), False)
    logit = logit[:, 0]
    logp, p = np.full(G, -np.inf), np.zeros(G)
    entropy, value = np.zeros(S), np.zeros(S)
    action = np.zeros(S, dtype=np.int32)
    zs = np.zeros((S, emb.shape[1]))
    for s in range(S):
        j0, j1 = int(sgp[s]), int(sgp[s + 1])
        valid = np.flatnonzero(mask[j0:j1]) + j0
        l = logit[valid]
        M = l.max()
        lse = M + np.log(np.exp(l - M).sum())
        logp[valid] = l - lse
        p[valid] = np.exp(l - lse)
        entropy[s] = -(p[valid] * logp[valid]).sum()
        action[s] = valid[np.flatnonzero(l == M)[0]] - j0
        zs[s] = emb[valid].mean(axis=0)
    v, c_v = mlp_forward(zs, _layers(W, "value"), False)
    value[:] = v[:, 0]
    return dict(logit=logit, logp=logp, p=p, entropy=entropy, action=action, value=value,
                z=zs, c_pi=c_pi, c_v=c_v)


# ----------------------------------------------------------------------------- backward
def _put(grads, model, prefix, g):
    for i, (dW, db) in enumerate(g):
        grads[f"{prefix}.W{i}"] += dW
        grads[f"{prefix}.b{i}"] += db


def zero_grads(model):
    return {name: np.zeros(shape, dtype=F) for name, shape in weight_layout(model)}


def policy_value_backward(model, w, emb, state, dlogp, dvalue, dentropy, bound=None, fw=None):
    """Gradient of L = sum_valid dlogp_j logp_j + sum_s dvalue_s value_s + sum_s dentropy_s
    entropy_s w.r.t. the embeddings [G, H] and the head weights (flat vector, zero elsewhere).
    Masked slots get exactly zero everywhere (invalid-action masking, Section 3.3.2).
    fw: the result of policy_value on the same arguments, if the caller already has it."""
    W = unflatten(model, w)
    if fw is None:
        fw = policy_value(model, w, emb, state)
    sgp, mask = state["state_graph_ptr"], np.asarray(state["slot_mask"]).astype(bool)
    S, G = len(sgp) - 1, emb.shape[0]
    dlogit = np.zeros(G)
    dz = np.zeros_like(fw["z"])
    dv = np.asarray(dvalue, dtype=F).reshape(S, 1)
    b_v, b_pi = ([], []) if bound is not None else (None, None)
    dzs, g_v = mlp_backward(dv, _layers(W, "value"), fw["c_v"], False, b_v)
    demb = np.zeros_like(np.asarray(emb, dtype=F))
    for s in range(S):
        j0, j1 = int(sgp[s]), int(sgp[s + 1])
        valid = np.flatnonzero(mask[j0:j1]) + j0
        c = np.asarray(dlogp, dtype=F)[valid]
        pv, lpv = fw["p"][valid], fw["logp"][valid]
        dlogit[valid] = c - pv * c.sum() - dentropy[s] * pv * (lpv + fw["entropy"][s])
        demb[valid] += dzs[s] / len(valid)
    dx, g_pi = mlp_backward(dlogit[:, None], _layers(W, "policy"), fw["c_pi"], False, b_pi)
    demb += dx          # rows of masked slots stay exactly zero: their dlogit is zero
    grads = zero_grads(model)
    _put(grads, model, "policy", g_pi)
    _put(grads, model, "value", g_v)
    if bound is not None:
        _put(bound, model, "policy", b_pi)
        _put(bound, model, "value", b_v)
    return demb, flatten(model, grads)


def _gat_round_backward(W, r, h, c, dh_out, src, dst, grads, bound=None):
    """Reverse of one graph-attention round (see encode_graph): h' = relu(pre),
    pre_i = sum_k alpha_k z[src_k] + alpha_i z_i with alpha the softmax over i's in-edges and its
    self edge of leaky(a_src . z_sender + a_dst . z_i), z = h W. Returns d/dh and accumulates the
    gradients of W, a_src, a_dst (and, into `bound`, their sums of absolute terms)."""
    Wg, a_s, a_d = W[f"gat{r}.W"], W[f"gat{r}.a_src"], W[f"gat{r}.a_dst"]
    z, alpha_e, alpha_s, pre = c["z"], c["alpha_e"], c["alpha_s"], c["pre"]
    n = h.shape[0]
    dpre = dh_out * (pre > 0.0)
    # through the weighted sum: to the summed rows, and to the weights
    dz = alpha_s[:, None] * dpre
    np.add.at(dz, src, alpha_e[:, None] * dpre[dst])
    dal_e = (dpre[dst] * z[src]).sum(axis=1)
    dal_s = (dpre * z).sum(axis=1)
    # softmax over each receiver's in-edges plus its self edge: ds = alpha (dalpha - sum alpha dalpha)
    tot = alpha_s * dal_s + segment_sum(alpha_e * dal_e, dst, n)
    ds_e = alpha_e * (dal_e - tot[dst])
    ds_s = alpha_s * (dal_s - tot)
    # leaky ReLU (slope 0.2) of u = a_src . z_sender + a_dst . z_receiver
    u_e = z[src] @ a_s + z[dst] @ a_d
    u_s = z @ a_s + z @ a_d
    du_e = ds_e * np.where(u_e > 0.0, 1.0, 0.2)
    du_s = ds_s * np.where(u_s > 0.0, 1.0, 0.2)
    d_ss = du_s + segment_sum(du_e, src, n)          # d / d (a_src . z_n): self edge + out-edges
    d_sd = du_s + segment_sum(du_e, dst, n)          # d / d (a_dst . z_n): self edge + in-edges
    grads[f"gat{r}.a_src"] += d_ss @ z
    grads[f"gat{r}.a_dst"] += d_sd @ z
    dz += d_ss[:, None] * a_s[None, :] + d_sd[:, None] * a_d[None, :]
    grads[f"gat{r}.W"] += h.T @ dz
    if bound is not None:
        bound[f"gat{r}.a_src"] += np.abs(d_ss) @ np.abs(z)
        bound[f"gat{r}.a_dst"] += np.abs(d_sd) @ np.abs(z)
        bound[f"gat{r}.W"] += np.abs(h).T @ np.abs(dz)
    return dz @ Wg.T


def encode_graph_backward(model, W, inter, demb_g, src, dst, grads, bound=None):
    """Accumulates into `grads` the gradient through one graph's encoder given d/d emb (and into
    `bound`, a dict like grads, the sums of absolute terms; see mlp_backward)."""
    def back(dy, prefix, cache):
        bl = [] if bound is not None else None
        dx, g = mlp_backward(dy, _layers(W, prefix), cache, True, bl)
        _put(grads, model, prefix, g)
        if bound is not None:
            _put(bound, model, prefix, bl)
        return dx
    n, H = inter["h"][0].shape[0], model["hidden"]
    dgin = back(np.asarray(demb_g, dtype=F)[None, :], "readout", inter["c_readout"])
    dpool = dgin[0, :H]
    if model["readout"] == "mean":
        dpool = dpool / max(n, 1)
    dh = np.tile(dpool, (n, 1))
    for r in reversed(range(model["rounds"])):
        if model.get("round_kind", "mlp") == "gat":
            dh = _gat_round_backward(W, r, inter["h"][r], inter["gat"][r], dh, src, dst, grads, bound)
            continue
        dxin = back(dh, f"node{r}", inter["c_node"][r])
        dh, dagg = dxin[:, :H].copy(), dxin[:, H:]
        dm = dagg[dst]                                   # reverse of the sum at the receiver
        dxe = back(dm, f"edge{r}", inter["c_edge"][r])
        np.add.at(dh, src, dxe[:, :H])                   # reverse of the gather by sender
        np.add.at(dh, dst, dxe[:, H:2 * H])              # reverse of the gather by receiver
    back(dh, "embed", inter["c_embed"])


def encode_backward(model, w, state, demb, graphs=None, bound=None):
    """Flat weight gradient (zero on head weights) of sum_g <demb_g, emb_g>. `bound`: optional
    dict from zero_grads() that receives the sums of absolute terms."""
    W = unflatten(model, w)
    grads = zero_grads(model)
    G = len(state["graph_node_ptr"]) - 1
    idx = range(G) if graphs is None else graphs
    for k, g in enumerate(idx):
        op, dense, src, dst, xe, gg = _graph_args(state, g)
        if gg is None:
            gg = np.zeros(model["d_global"])
        inter = encode_graph(model, W, op, dense, src, dst, xe, gg)
        encode_graph_backward(model, W, inter, demb[k], src, dst, grads, bound)
    return flatten(model, grads)


def loss_and_grad(model, w, state, dlogp, dvalue, dentropy, bound=None):
    """L (see policy_value_backward) and dL/dw through heads and encoder."""
    emb = encode(model, w, state)
    fw = policy_value(model, w, emb, state)
    valid = np.asarray(state["slot_mask"]).astype(bool)
    L = (np.asarray(dlogp, dtype=F)[valid] * fw["logp"][valid]).sum() \
        + (np.asarray(dvalue, dtype=F) * fw["value"]).sum() \
        + (np.asarray(dentropy, dtype=F) * fw["entropy"]).sum()
    demb, gh = policy_value_backward(model, w, emb, state, dlogp, dvalue, dentropy, bound)
    return L, gh + encode_backward(model, w, state, demb, bound=bound), demb


# ----------------------------------------------------------------------------- objective
def ppo_objective(logp, value, entropy, state, action, old_logp, advantage, v_target,
                  eps=0.2, c1=0.5, c2=0.01):
    """Clipped-surrogate objective of Section 3.3.4 (to be minimised) over the S states of a
    minibatch, from the heads' outputs:
      ratio_s  = exp(logp[slot of the action taken in s] - old_logp_s)
      L_clip   = -mean_s min(ratio_s A_s, clip(ratio_s, 1-eps, 1+eps) A_s)      (first equation)
      L_vf     =  mean_s (value_s - v_target_s)^2                               (second equation)
      L_ent    = -mean_s entropy_s          (the entropy term enters as a bonus)
      J        = L_clip + c1 L_vf + c2 L_ent                                    (third equation)
    `action` is the slot index inside each state (0 = No-Op). eps is not printed in the paper
    (a parameter; 0.2 is the PPO paper's default). Returns J, its three parts and dJ/dlogp [G],
    dJ/dvalue [S], dJ/dentropy [S] (the inputs of policy_value_backward). Where both arguments of
    the min are equal the unclipped one is differentiated."""
    sgp = np.asarray(state["state_graph_ptr"])
    S, G = len(sgp) - 1, len(np.asarray(logp))
    logp, value, entropy = (np.asarray(x, dtype=F) for x in (logp, value, entropy))
    old_logp, A, vt = (np.asarray(x, dtype=F) for x in (old_logp, advantage, v_target))
    slot = sgp[:-1] + np.asarray(action)
    ratio = np.exp(logp[slot] - old_logp)
    s1 = ratio * A
    s2 = np.clip(ratio, 1.0 - eps, 1.0 + eps) * A
    l_clip = -np.minimum(s1, s2).mean() if S else 0.0
    l_vf = ((value - vt) ** 2).mean() if S else 0.0
    l_ent = -entropy.mean() if S else 0.0
    dlogp = np.zeros(G)
    dlogp[slot] = np.where(s1 <= s2, -s1, 0.0) / max(S, 1)       # d(ratio A)/dlogp = ratio A
    dvalue = 2.0 * c1 * (value - vt) / max(S, 1)
    dentropy = np.full(S, -c2 / max(S, 1))
    return dict(J=l_clip + c1 * l_vf + c2 * l_ent, l_clip=l_clip, l_vf=l_vf, l_ent=l_ent,
                dlogp=dlogp, dvalue=dvalue, dentropy=dentropy)
