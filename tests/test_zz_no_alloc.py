"""xrl_policy_value_static, the entry point that allocates nothing, against xrl_policy_value.

Both run the same single-launch kernel, so every output must be bit-identical. Two calls in a row
share the GPU's fixed scratch array, the second on a smaller batch (stale counters, logits and
mean embeddings of the first call must not leak into it). Sizes beyond the fixed scratch are
rejected before anything is launched.
"""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def heads_state(rng, model, n_states, n_cand):
    slots = np.concatenate([[1], rng.integers(2, n_cand + 2, n_states - 1)]).astype(np.int64)[:n_states]
    G = int(slots.sum())
    sgp = np.concatenate([[0], np.cumsum(slots)]).astype(np.int32)
    mask = (rng.random(G) > 0.3).astype(np.uint8)
    mask[sgp[:-1]] = 1
    return dict(n_states=n_states, state_graph_ptr=sgp,
                graph_node_ptr=np.arange(G + 1, dtype=np.int32), graph_edge_ptr=np.zeros(G + 1, np.int32),
                node_op=rng.integers(0, model["n_op_types"], G).astype(np.int32),
                node_dense=rng.integers(0, 13, (G, model["n_node_dense"])).astype(np.float32),
                edge_src=np.zeros(0, np.int32), edge_dst=np.zeros(0, np.int32),
                edge_feat=np.zeros((0, model["d_edge"]), np.float32),
                graph_global=np.zeros((G, model["d_global"]), np.float32), slot_mask=mask)


@pytest.mark.parametrize("hidden", [64, 256])
def test_static_entry_point_equals_allocating_one(hidden):
    import torch
    import paper_2304_14698_amd as xrl
    xrl.load_library()
    rng = np.random.Generator(np.random.PCG64(2304))
    model, _ = synth.make_config(1)
    model.update(hidden=hidden, rounds=1)
    w = synth.init_weights(rng, xrl.weight_layout(model), bias_range=0.1)
    enc = xrl.Encoder(model, w)
    # first a batch of many states, then a smaller one: stale scratch contents must not matter
    for n_states, n_cand in [(40, 90), (5, 12)]:
        state = heads_state(rng, model, n_states, n_cand)
        batch = enc.pack(state)
        G, S = batch.G, batch.S
        assert G <= 4096 and S * hidden <= 65536
        emb = torch.from_numpy(rng.standard_normal((G, hidden)).astype(np.float32)).cuda()
        ref = enc.policy_value(batch, emb)
        torch.cuda.synchronize()
        for with_logit in (True, False):
            out = dict(logp=torch.full((G,), 7.0, device="cuda"), value=torch.full((S,), 7.0, device="cuda"),
                       entropy=torch.full((S,), 7.0, device="cuda"),
                       action=torch.full((S,), -7, dtype=torch.int32, device="cuda"))
            if with_logit:
                out["logit"] = torch.full((G,), 7.0, device="cuda")
            enc.policy_value(batch, emb, out=out, static=True)
            torch.cuda.synchronize()
            for k in out:
                assert torch.equal(out[k], ref[k]), f"{k} differs (states {n_states}, logit buffer {with_logit})"
        batch.free()
    # beyond the fixed scratch: refused with a clear error, outputs untouched
    big = heads_state(rng, model, 90, 150)
    batch = enc.pack(big)
    assert batch.G > 4096
    emb = torch.zeros((batch.G, hidden), device="cuda")
    out = dict(logp=torch.full((batch.G,), 7.0, device="cuda"), value=torch.full((batch.S,), 7.0, device="cuda"),
               entropy=torch.full((batch.S,), 7.0, device="cuda"),
               action=torch.full((batch.S,), -7, dtype=torch.int32, device="cuda"))
    with pytest.raises(xrl.XrlError) as ei:
        enc.policy_value(batch, emb, out=out, static=True)
    assert ei.value.code == xrl.ERR["UNSUPPORTED"] and "4096" in str(ei.value)
    torch.cuda.synchronize()
    assert float(out["logp"].min()) == 7.0
    batch.free()
    enc.close()
