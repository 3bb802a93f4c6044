"""The weight-gradient product dW = X^T dZ, db = 1^T dZ of the encoder's backward on its own,
against float64 on the same operand values, through the C ABI.

The backward parity tests of the bf16 path can only use per-tensor criteria (ReLU masks taken from
a bf16 forward differ from the float64 oracle's); a gradient kernel that dropped a few rows would
pass them. Here the operands are given -- values exactly representable in the operand type -- so
the only difference from float64 is the fp32 accumulation:  |got - ref| <= 2e-6 B + 1e-30, with
B = |X|^T |dZ| the sum of the absolute terms of an entry (fp32 partial sums over a few thousand
rows; measured below 3e-7 B). Exact zeros where X has a zero column. Every call is repeated: the
result must be bit-identical (fixed summation order)."""
import numpy as np
import pytest

import synth
from test_gpu_forward import weights_for

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xrl():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2304_14698_amd as x
    x.load_library()
    return x


def operand(rng, shape, precision, scale=1.0):
    """Random values exactly representable in the operand type, as (float64 array, device tensor)."""
    import torch
    a = torch.from_numpy((rng.standard_normal(shape) * scale).astype(np.float32))
    a = a.to(torch.bfloat16) if precision == "bf16" else a
    return a.to(torch.float64).numpy(), a.cuda()


def run(xrl, model, state, kinds=("plain", "edge", "node"), n_plain=None):
    import torch
    prec, H, De = model["precision"], model["hidden"], model["d_edge"]
    rng = np.random.Generator(np.random.PCG64(77))
    enc = xrl.Encoder(model, weights_for(model))
    batch = enc.pack(state)
    v = batch.host_view()
    N, E = batch.N, batch.E
    h64, h = operand(rng, (N, H), prec)
    agg64, agg = operand(rng, (N, H), prec)
    # the sums' rows of nodes without in-edges count as zero and are not read (the forward never
    # writes them): poisoned on the device
    no_in = np.diff(v["in_ptr"]) == 0
    agg64[no_in] = 0.0
    agg[torch.from_numpy(no_in).cuda()] = float("nan")
    feat = v["edge_feat"].astype(np.float32)
    if prec == "bf16":
        feat = torch.from_numpy(feat).to(torch.bfloat16).to(torch.float32).numpy()   # as the kernel rounds them
    for kind in kinds:
        rows = {"plain": n_plain or E, "edge": E, "node": N}[kind]
        dz64, dz = operand(rng, (rows, H), prec, 0.5)
        if kind == "plain":
            x64, x = operand(rng, (rows, H), prec)
            X, args = x64, dict(x=x)
        elif kind == "edge":
            X = np.concatenate([h64[v["in_src"]], h64[v["in_dst"]], feat.astype(np.float64)], axis=1)
            args = dict(x=h)
        else:
            X = np.concatenate([h64, agg64], axis=1)
            args = dict(x=h, x2=agg)
        K = X.shape[1]
        ref_w, ref_b = X.T @ dz64, dz64.sum(axis=0)
        B_w, B_b = np.abs(X).T @ np.abs(dz64), np.abs(dz64).sum(axis=0)
        out = []
        for _ in range(2):
            dW = torch.zeros((K, H), dtype=torch.float32, device="cuda")
            db = torch.zeros(H, dtype=torch.float32, device="cuda")
            enc.weight_gradient(batch, kind, dz=dz, dW=dW, db=db, **args)
            torch.cuda.synchronize()
            out.append((dW.clone(), db.clone()))
        assert torch.equal(out[0][0], out[1][0]) and torch.equal(out[0][1], out[1][1]), f"{kind}: two calls differ"
        gw, gb = out[0][0].cpu().numpy().astype(np.float64), out[0][1].cpu().numpy().astype(np.float64)
        ew, eb = np.abs(gw - ref_w) - (2e-6 * B_w + 1e-30), np.abs(gb - ref_b) - (2e-6 * B_b + 1e-30)
        assert ew.max() <= 0, (kind, H, prec, "dW", float((np.abs(gw - ref_w) / (B_w + 1e-30)).max()))
        assert eb.max() <= 0, (kind, H, prec, "db", float((np.abs(gb - ref_b) / (B_b + 1e-30)).max()))
        # accumulation into the caller's buffers
        enc.weight_gradient(batch, kind, dz=dz, dW=out[0][0], db=out[0][1], **args)
        torch.cuda.synchronize()
        np.testing.assert_allclose(out[0][0].cpu().numpy(), 2 * gw, rtol=1e-6, atol=1e-6 * np.abs(gw).max())
    batch.free()
    enc.close()


@pytest.mark.parametrize("hidden,precision", [(64, "bf16"), (128, "bf16"), (256, "bf16"), (128, "fp32")])
def test_weight_gradient_product(xrl, hidden, precision):
    model, state = synth.make_config(4, n_cand=3)            # ~5000 rows, ragged against every tile size
    model.update(hidden=hidden, precision=precision)
    run(xrl, model, state, n_plain=4097)


@pytest.mark.parametrize("hidden", [128, 256])
def test_weight_gradient_product_wide_tiles(xrl, hidden, monkeypatch):
    """The 256-column tiles (used from 2^20 rows on), forced onto the same small batch."""
    monkeypatch.setenv("XRL_WGRAD_WIDE_MIN_ROWS", "0")
    model, state = synth.make_config(4, n_cand=3)
    model.update(hidden=hidden, precision="bf16")
    run(xrl, model, state, n_plain=3001)


def test_weight_gradient_product_few_rows_and_hubs(xrl):
    """Fewer rows than one stage, and the paper's feature dimensions (4 edge attributes)."""
    model, state = synth.make_config(1)
    model.update(hidden=128, precision="bf16", d_edge=4)
    state = dict(state, edge_feat=np.ascontiguousarray(state["edge_feat"][:, :4]))
    run(xrl, model, state, n_plain=7)
