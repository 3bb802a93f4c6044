"""Helpers of the GPU gradient-parity tests: element-wise criteria against the float64 oracle.

fp32 criterion, per weight tensor and element-wise (scale = max|ref| of the tensor, floored at
1e-3 of the largest gradient entry overall; B = sum over rows of |x| |dz| for that entry, the sum
of the absolute terms the entry is made of, returned by the oracle):
    |g - ref| <= 1e-5 |ref| + 1e-5 scale + 2e-6 B + A
  * 1e-5 relative and 1e-5 of the tensor's scale are the fp32 tolerance of the forward path;
  * 2e-6 B is the rounding error of the sum itself: every term carries the relative error of two
    fp32 factors that each went through a few dozen fp32 operations (about 1e-6), and the sum is
    taken in fp32; the weight-gradient product on exactly representable operands is held to the
    same 2e-6 B in test_gpu_weight_gradient.py;
  * A is non-zero only where the oracle itself says a ReLU mask is undecided: a pre-activation
    within 1e-5 of its layer's scale of zero (the forward's tolerance) may take either mask on the
    GPU. For every such pre-activation the oracle's reverse mode is run once more on that graph
    with the mask inverted (by negating the cached pre-activation, which the reverse mode only
    uses for the mask), and A = sum over them of |change of the gradient|.

bf16 criterion on mask-stable cases (every pre-activation of the oracle at least `margin` away
from zero, asserted, so that both sides differentiate the same piecewise-linear function):
  * all units on, non-negative weights, attributes and upstream gradients: no term of any sum
    cancels, and the stated tolerance holds as it is: |g - ref| <= 2e-2 |ref| + 1e-3 scale;
  * units on or off per feature, weights and upstream gradients of both signs:
        |g - ref| <= 2e-2 |ref| + 1e-3 scale + 4e-5 C
    C = the same gradient entry evaluated by the oracle's reverse mode with every weight, input
    and upstream gradient replaced by its absolute value (same masks): the sum of the absolute
    values of all the terms the entry is made of, through the whole chain of layers. Every stored
    gradient between the loss and a weight is rounded to bf16 (2^-9) and is a sum that cancels;
    C is what those roundings are proportional to in the worst case. Products of absolute values
    through a dozen layers do not cancel at all, so C overstates the typical error by far: the
    factor is measurement times three (largest (error - the first two terms) / C over the cases
    of test_gpu_backward.py: 1.3e-5, printed by the tests), which puts the last term at about a
    hundredth of a tensor's scale.
  The same cases pass the fp32 criterion in fp32 with no allowance, so what the bf16 runs add is
  rounding, not arithmetic.

In the chained test (heads + encoder) the first layer of each head also gets 1e-5 max|emb| times the
bound of its bias gradient (sum over rows of |dz|): the embeddings it multiplies carry the forward's
absolute error. Hidden units of the heads within 1e-5 of zero are treated like the encoder's
(heads_flip_allowance).

Heads (fp32 in both modes), on given embeddings: |g - ref| <= 1e-5 |ref| + 1e-5 scale + kappa B
with kappa = 2e-6 + 1e-5 max(1, L), L = the largest |logit|: the forward's tolerance admits an
absolute error of 1e-5 L in logp (a difference of logits), i.e. a relative error of 1e-5 L in every
probability, and the heads' gradients are linear in the probabilities.
"""
import numpy as np

from oracle import xrl_oracle as O


def tensors(om):
    o = 0
    for name, shape in O.weight_layout(om):
        n = int(np.prod(shape))
        yield name, slice(o, o + n), shape
        o += n


def _caches(model, inter):
    """(prefix, layer, z array) of every ReLU of one graph's encoder forward."""
    out = [("embed", l, c) for l, c in enumerate(inter["c_embed"])]
    out += [("readout", l, c) for l, c in enumerate(inter["c_readout"])]
    for r, cs in enumerate(inter["c_edge"]):
        out += [(f"edge{r}", l, c) for l, c in enumerate(cs)]
    for r, cs in enumerate(inter["c_node"]):
        out += [(f"node{r}", l, c) for l, c in enumerate(cs)]
    return out


def min_margin(om, w, state, graphs=None):
    """Smallest |pre-activation| over every ReLU of the encoder (the oracle's caches) and the
    share of units that are on."""
    W = O.unflatten(om, w)
    G = len(state["graph_node_ptr"]) - 1
    lo, on, cnt = np.inf, 0, 0
    for g in (range(G) if graphs is None else graphs):
        op, dense, src, dst, xe, gg = O._graph_args(state, g)
        inter = O.encode_graph(om, W, op, dense, src, dst, xe, gg if gg is not None else np.zeros(om["d_global"]))
        for _, _, (x, z) in _caches(om, inter):
            if z.size:
                lo = min(lo, float(np.abs(z).min()))
                on += int((z > 0).sum())
                cnt += z.size
    return lo, on / max(cnt, 1)


def flip_allowance(om, w, state, demb, eps=1e-5, graphs=None, max_flips=4000):
    """A (see the module docstring) for upstream embedding gradients demb [len(graphs), H], and the
    number of undecided pre-activations."""
    W = O.unflatten(om, w)
    G = len(state["graph_node_ptr"]) - 1
    A = np.zeros(O.weight_count(om))
    n_near = 0
    for k, g in enumerate(range(G) if graphs is None else graphs):
        op, dense, src, dst, xe, gg = O._graph_args(state, g)
        inter = O.encode_graph(om, W, op, dense, src, dst, xe, gg if gg is not None else np.zeros(om["d_global"]))
        near = []
        if om.get("round_kind", "mlp") == "gat":
            zs = [c["pre"] for c in inter["gat"]] + [z for _, _, (x, z) in _caches(om, inter)]
        else:
            zs = [z for _, _, (x, z) in _caches(om, inter)]
        for z in zs:
            if z.size:
                idx = np.argwhere(np.abs(z) <= eps * max(1.0, float(np.abs(z).max())))
                near += [(z, tuple(i)) for i in idx]
        if not near:
            continue
        n_near += len(near)
        assert n_near <= max_flips, "too many undecided ReLU masks for the per-mask allowance"
        base = O.zero_grads(om)
        O.encode_graph_backward(om, W, inter, demb[k], src, dst, base)
        base = O.flatten(om, base)
        for z, i in near:
            old = z[i]
            z[i] = -old if old != 0.0 else 1e-300
            gr = O.zero_grads(om)
            O.encode_graph_backward(om, W, inter, demb[k], src, dst, gr)
            A += np.abs(O.flatten(om, gr) - base)
            z[i] = old
    return A, n_near


def heads_flip_allowance(om, w, emb, state, dlogp, dvalue, dentropy, eps=1e-5, max_flips=200):
    """The same allowance for the heads' own ReLUs (their hidden layers), on the head tensors: for
    every hidden pre-activation of the policy or value head that the oracle has within eps of its
    layer's scale of zero, the heads' reverse mode is run with that mask inverted, and the
    absolute changes of the head gradients are summed. Returns (A, number of such units)."""
    fw = O.policy_value(om, w, emb, state)
    base = O.policy_value_backward(om, w, emb, state, dlogp, dvalue, dentropy, fw=fw)[1]
    A = np.zeros_like(base)
    n_near = 0
    for key in ("c_pi", "c_v"):
        for x, z in fw[key][:-1]:                      # (the last layer of a head has no ReLU)
            if not z.size:
                continue
            for i in np.argwhere(np.abs(z) <= eps * max(1.0, float(np.abs(z).max()))):
                i = tuple(i)
                n_near += 1
                assert n_near <= max_flips, "too many undecided ReLU masks in the heads"
                old = z[i]
                z[i] = -old if old != 0.0 else 1e-300
                A += np.abs(O.policy_value_backward(om, w, emb, state, dlogp, dvalue, dentropy, fw=fw)[1] - base)
                z[i] = old
    return A, n_near


def check_fp32(got, ref, bound, om, allowance=None, only=None, kappa=2e-6, atol=1e-5):
    bad = []
    gscale = float(np.abs(ref).max())
    for name, sl, _ in tensors(om):
        if only is not None and not name.startswith(only):
            continue
        g, r, B = got[sl].astype(np.float64), ref[sl], bound[sl]
        scale = max(float(np.abs(r).max()), 1e-3 * gscale)
        tol = 1e-5 * np.abs(r) + atol * scale + kappa * B
        if allowance is not None:
            tol = tol + allowance[sl]
        err = np.abs(g - r) - tol
        if np.any(err > 0):
            i = int(np.argmax(err))
            bad.append(f"{name}: {(err > 0).sum()}/{g.size} outside tolerance, worst [{i}] got {g[i]:.9g} "
                       f"ref {r[i]:.9g} scale {scale:.3g} B {B[i]:.3g} tol {tol[i]:.3g}; first indices "
                       f"{np.flatnonzero(err > 0)[:12].tolist()}, largest (error - other terms) / B "
                       f"{float(((np.abs(g - r) - (tol - kappa * B)) / np.maximum(B, 1e-300)).max()):.3g}")
    assert not bad, "\n".join(bad)


def abs_chain_bound(om, w, state, demb, graphs=None):
    """C of the module docstring: the oracle's encoder reverse mode on absolute values (weights,
    cached layer inputs, upstream gradient), masks as in the real forward."""
    W = O.unflatten(om, w)
    Wabs = {k: np.abs(v) for k, v in W.items()}
    G = len(state["graph_node_ptr"]) - 1
    grads = O.zero_grads(om)
    for k, g in enumerate(range(G) if graphs is None else graphs):
        op, dense, src, dst, xe, gg = O._graph_args(state, g)
        inter = O.encode_graph(om, W, op, dense, src, dst, xe, gg if gg is not None else np.zeros(om["d_global"]))
        for key in ("c_embed", "c_readout"):
            inter[key] = [(np.abs(x), z) for x, z in inter[key]]
        for key in ("c_edge", "c_node"):
            inter[key] = [[(np.abs(x), z) for x, z in c] for c in inter[key]]
        O.encode_graph_backward(om, Wabs, inter, np.abs(demb[k]), src, dst, grads)
    return O.flatten(om, grads)


def check_bf16_elementwise(got, ref, om, chain_bound=None, factor=4e-5):
    """The bf16 criterion (module docstring); returns the largest (error - first two terms) / C."""
    bad, worst = [], 0.0
    for name, sl, _ in tensors(om):
        if name.startswith(("policy", "value")):
            continue
        g, r = got[sl].astype(np.float64), ref[sl]
        scale = float(np.abs(r).max())
        tol = 2e-2 * np.abs(r) + 1e-3 * scale
        if chain_bound is not None:
            C = chain_bound[sl]
            worst = max(worst, float(((np.abs(g - r) - tol) / np.maximum(C, 1e-300)).max()))
            tol = tol + factor * C
        err = np.abs(g - r) - tol
        if np.any(err > 0):
            i = int(np.argmax(err))
            bad.append(f"{name}: {(err > 0).sum()}/{g.size} outside tolerance, worst [{i}] got {g[i]:.6g} "
                       f"ref {r[i]:.6g} scale {scale:.3g}" + (f" C {chain_bound[sl][i]:.3g}" if chain_bound is not None else ""))
    assert not bad, "\n".join(bad)
    return worst


def stable_weights(om, kind, seed, max_indeg=8, max_nodes=1500):
    """Weights under which no ReLU mask of the encoder depends on rounding.
    kind "all_on": non-negative matrices (a quarter of the entries non-zero), positive biases; with
      non-negative attributes every pre-activation is at least its bias, so every unit is on.
    kind "fixed": biases of magnitude 1.5..2.5 with random signs and matrices a tenth of the
      Glorot range (rows that multiply a sum over in-edges or over a graph's nodes scaled down by
      the largest in-degree / graph size), so a unit is on or off for every row alike; the
      one-hot rows of the node-update layer are +-3 with a zero bias, so its first layer's units
      are on or off by operator type. The margin is asserted by the caller (min_margin)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    De, T, H = om["d_edge"], om["n_op_types"], om["hidden"]
    parts = []
    for name, shape in O.weight_layout(om):
        head = name.startswith(("policy", "value"))
        if len(shape) == 2:
            a = np.sqrt(6.0 / (shape[0] + shape[1]))
            if head:
                Wm = rng.uniform(-a, a, size=shape)
            elif kind == "all_on":
                Wm = rng.uniform(0, 8.0 / shape[0], size=shape) * (rng.random(shape) < 0.25)
            else:
                Wm = rng.uniform(-a, a, size=shape) * 0.1
                if name == "embed.W0":
                    Wm[De:De + T] = rng.choice([-3.0, 3.0], size=(T, shape[1]))
                    Wm[:De] /= max_indeg
                elif name.startswith("node") and name.endswith("W0"):
                    Wm[H:] /= max_indeg
                elif name == "readout.W0":
                    Wm[:H] /= max_nodes
            parts.append(Wm.astype(np.float32).ravel())
        else:
            if head:
                b = rng.uniform(-0.1, 0.1, size=shape)
            elif kind == "all_on":
                b = rng.uniform(0.05, 0.15, size=shape)
            elif name == "embed.b0":
                b = np.zeros(shape)
            else:
                b = rng.choice([-1.0, 1.0], size=shape) * rng.uniform(1.5, 2.5, size=shape)
            parts.append(b.astype(np.float32).ravel())
    return np.concatenate(parts)
