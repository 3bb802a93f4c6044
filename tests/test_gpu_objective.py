"""GPU parity of the clipped-surrogate objective (Section 3.3.4) against the oracle, through the C
ABI: the objective's own outputs elementwise (fp32 arithmetic on a handful of numbers per state:
rtol 1e-5, atol 1e-6), then the whole update chain -- objective -> heads backward -> encoder
backward -- against the oracle's chain on the same inputs, to the fp32 gradient criterion of
test_gpu_backward.py."""
import numpy as np
import pytest

import synth
from oracle import xrl_oracle as O
from test_gpu_forward import oracle_model, weights_for
from test_gpu_backward import check_grads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xrl():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2304_14698_amd as x
    x.load_library()
    return x


def rollout_records(rng, state, logp):
    """Seeded stand-ins for what a rollout stores: a valid action per state, the log-probability it
    had under a slightly different (older) policy, advantages, value targets."""
    sgp, mask = np.asarray(state["state_graph_ptr"]), np.asarray(state["slot_mask"]).astype(bool)
    S = len(sgp) - 1
    action = np.array([rng.choice(np.flatnonzero(mask[sgp[s]:sgp[s + 1]])) for s in range(S)], np.int32)
    slot = sgp[:-1] + action
    old = (logp[slot] + 0.3 * rng.standard_normal(S)).astype(np.float32)     # ratios inside and outside the clip range
    return action, old, rng.standard_normal(S).astype(np.float32), rng.standard_normal(S).astype(np.float32)


@pytest.mark.parametrize("cfg,n_states", [(1, None), (3, 6)])
def test_objective_and_update_chain(xrl, cfg, n_states):
    import torch
    model, state = synth.make_config(cfg, n_states=n_states, n_cand=6 if cfg == 3 else None)
    model["precision"] = "fp32"
    w = weights_for(model)
    om = oracle_model(model)
    enc = xrl.Encoder(model, w)
    batch = enc.pack(state)
    emb = enc.encode(batch, save_for_backward=True)
    pv = enc.policy_value(batch, emb)
    torch.cuda.synchronize()
    rng = np.random.Generator(np.random.PCG64(77 + cfg))
    logp = pv["logp"].cpu().numpy().astype(np.float64)
    action, old, adv, vt = rollout_records(rng, state, logp)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    eps, c1, c2 = 0.2, 0.5, 0.01
    J, dlogp, dvalue, dentropy = enc.ppo_objective(batch, pv, t(action), t(old), t(adv), t(vt), eps, c1, c2)
    torch.cuda.synchronize()
    # the objective itself, on the GPU's own head outputs
    ref = O.ppo_objective(logp, pv["value"].cpu().numpy(), pv["entropy"].cpu().numpy(), state, action, old, adv, vt,
                          eps, c1, c2)
    ratio = np.exp(logp[np.asarray(state["state_graph_ptr"])[:-1] + action] - old)
    assert (np.abs(ratio - (1 - eps)) > 1e-4).all() and (np.abs(ratio - (1 + eps)) > 1e-4).all(), "seed sits on a kink"
    np.testing.assert_allclose(J.cpu().numpy(), [ref["J"], ref["l_clip"], ref["l_vf"], ref["l_ent"]], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(dlogp.cpu().numpy(), ref["dlogp"], rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose(dvalue.cpu().numpy(), ref["dvalue"], rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose(dentropy.cpu().numpy(), ref["dentropy"], rtol=1e-5, atol=1e-9)
    # the update chain: gradient of J w.r.t. every weight
    dw = torch.zeros(enc.n_weights, dtype=torch.float32, device="cuda")
    demb = enc.policy_value_backward(batch, emb, dlogp, dvalue, dentropy, dw)
    enc.encode_backward(batch, demb, dw)
    torch.cuda.synchronize()
    emb64 = O.encode(om, w, state)
    fw = O.policy_value(om, w, emb64, state)
    r64 = O.ppo_objective(fw["logp"], fw["value"], fw["entropy"], state, action, old, adv, vt, eps, c1, c2)
    assert abs(float(J[0]) - r64["J"]) <= 1e-4 * max(1.0, abs(r64["J"]))
    bound = O.zero_grads(om)
    _, ref_dw, _ = O.loss_and_grad(om, w, state, r64["dlogp"], r64["dvalue"], r64["dentropy"], bound=bound)
    check_grads(dw.cpu().numpy(), ref_dw, O.flatten(om, bound), model)
    batch.free()
    enc.close()
