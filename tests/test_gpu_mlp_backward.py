"""One backward step through a fused two-layer MLP of a message-passing round (xrl_mlp_backward)
against float64 on the same operand values, through the C ABI.

Weights and inputs are exactly representable in the operand type, and the float64 reference rounds
where the kernel does (z1 and dz1 become operands of the next product in the operand type; edge
attributes enter as operands), and takes each stage's input as the kernel stored it (dx is checked as the product of the stored
dz1), so what is left is the fp32 accumulation and one final rounding of each stored value: |got - ref| <= 2^-7 |ref| + 1e-4 max|ref| for bf16 (one unit in the last place),
1e-5 |ref| + 1e-5 max|ref| for fp32. A row is compared only if none of its pre-activations lies
within 2e-5 of zero relative to the tensor's scale: there the ReLU mask may legitimately differ
(at most a fifth of the rows may be set aside this way). The end-to-end bf16 criteria cannot be
this tight because their masks come from a bf16 forward."""
import numpy as np
import pytest

import synth
from oracle import xrl_oracle as O
from test_gpu_forward import oracle_model, weights_for

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xrl():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2304_14698_amd as x
    x.load_library()
    return x


def rnd(a, precision):
    """float64 array rounded to the operand type (bf16: round to nearest even, as the kernels do)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if precision == "bf16":
        t = t.to(torch.bfloat16)
    return t.to(torch.float64).numpy()


def dev(a, precision):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return (t.to(torch.bfloat16) if precision == "bf16" else t).cuda()


def close(got, ref, rows_ok, precision, what):
    g = got.to(__import__("torch").float64).cpu().numpy()[rows_ok]
    r = rnd(ref, precision)[rows_ok]
    rtol, atol = (2.0 ** -7, 1e-4) if precision == "bf16" else (1e-5, 1e-5)
    err = np.abs(g - r) - (rtol * np.abs(r) + atol * np.abs(r).max())
    assert err.max() <= 0, (what, int((err > 0).sum()), err.size, float(np.abs(g - r).max()), float(np.abs(r).max()))


@pytest.mark.parametrize("hidden,precision", [(64, "bf16"), (128, "bf16"), (256, "bf16"), (128, "fp32")])
def test_mlp_backward_step(xrl, hidden, precision):
    import torch
    model, state = synth.make_config(4, n_cand=3)
    model.update(hidden=hidden, precision=precision, rounds=2)
    H, De = hidden, model["d_edge"]
    om = oracle_model(model)
    w = rnd(weights_for(model), precision).astype(np.float32)          # weights exact in the operand type
    W = O.unflatten(om, w.astype(np.float64))
    enc = xrl.Encoder(model, w)
    batch = enc.pack(state)
    v = batch.host_view()
    N, E = batch.N, batch.E
    rng = np.random.Generator(np.random.PCG64(41))
    h = rnd(rng.standard_normal((N, H)) * 0.7, precision)
    agg = rnd(rng.standard_normal((N, H)) * 0.7, precision)
    dy = rnd(rng.standard_normal((N, H)) * 0.3, precision)
    for kind, r in (("edge", 1), ("node", 0)):
        pre = f"{kind}{r}"
        W1, b1, W2, b2 = W[f"{pre}.W0"], W[f"{pre}.b0"], W[f"{pre}.W1"], W[f"{pre}.b1"]
        if kind == "edge":
            x = np.concatenate([h[v["in_src"]], h[v["in_dst"]], rnd(v["edge_feat"], precision)], axis=1)
            up = dy[v["in_dst"]]
        else:
            x = np.concatenate([h, agg], axis=1)
            up = dy
        pre1 = x @ W1 + b1
        z1 = np.maximum(pre1, 0.0)
        z1o = rnd(z1, precision)
        y = z1o @ W2 + b2
        dz2 = up * (y > 0)
        d1 = (dz2 @ W2.T) * (pre1 > 0)
        args = dict(h=dev(h, precision), dy=dev(dy, precision))
        if kind == "node":
            args.update(agg=dev(agg, precision), y=dev(np.maximum(y, 0.0), precision))
            yk = rnd(np.maximum(y, 0.0), precision)               # the kernel sees the stored (rounded) output
            dz2 = up * (yk > 0)
            d1 = (dz2 @ W2.T) * (pre1 > 0)
        out = enc.mlp_backward(batch, kind, r, **args)
        torch.cuda.synchronize()
        eps1, eps2 = 2e-5 * np.abs(pre1).max(), 2e-5 * np.abs(y).max()
        rows_ok = (np.abs(pre1) > eps1).all(axis=1) & (np.abs(y) > eps2).all(axis=1)
        assert rows_ok.mean() > 0.8, rows_ok.mean()
        close(out["z1"], z1, np.ones(len(z1), bool), precision, f"{kind} z1")
        close(out["dz2"], dz2, rows_ok, precision, f"{kind} dz2")
        close(out["dz1"], d1, rows_ok, precision, f"{kind} dz1")
        # dx is a product of the dz1 the kernel stored: a last-place difference in dz1, allowed
        # above, would otherwise count again here
        dx = out["dz1"].to(torch.float64).cpu().numpy() @ W1[:2 * H].T
        close(out["dxa"], dx[:, :H], rows_ok, precision, f"{kind} dx (first part)")
        close(out["dxb"], dx[:, H:], rows_ok, precision, f"{kind} dx (second part)")
    batch.free()
    enc.close()
