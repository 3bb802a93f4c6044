"""GPU parity of the clipped-surrogate objective (Section 3.3.4) against the oracle, through the C
ABI: the GPU's chain forward -> objective -> heads backward -> encoder backward against the
oracle's own chain on the same state, weights and rollout records (nothing the oracle takes comes
from the GPU): the objective's outputs element-wise at the tolerance its input logp carries, the
weight gradients to the chain criterion of test_gpu_backward.py."""
import numpy as np
import pytest

import synth
from oracle import xrl_oracle as O
from test_gpu_forward import oracle_model, weights_for
import grad_checks as GC
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
    # the oracle's own chain: forward, objective, reverse mode. The rollout's records are drawn
    # around the oracle's log-probabilities; the GPU gets the same records.
    emb64 = O.encode(om, w, state)
    fw = O.policy_value(om, w, emb64, state)
    L = max(1.0, float(np.abs(fw["logit"]).max()))
    rng = np.random.Generator(np.random.PCG64(77 + cfg))
    action, old, adv, vt = rollout_records(rng, state, fw["logp"])
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    eps, c1, c2 = 0.2, 0.5, 0.01
    J, dlogp, dvalue, dentropy = enc.ppo_objective(batch, pv, t(action), t(old), t(adv), t(vt), eps, c1, c2)
    torch.cuda.synchronize()
    r64 = O.ppo_objective(fw["logp"], fw["value"], fw["entropy"], state, action, old, adv, vt, eps, c1, c2)
    ratio = np.exp(fw["logp"][np.asarray(state["state_graph_ptr"])[:-1] + action] - old)
    assert (np.abs(ratio - (1 - eps)) > 1e-3).all() and (np.abs(ratio - (1 + eps)) > 1e-3).all(), "seed sits on a kink"
    # logp carries an absolute error of up to 1e-5 L (the forward's tolerance; L = largest |logit|),
    # so the probability ratio, and with it L_clip and dlogp, a relative one of 1e-5 L
    rt = 1e-5 + 1e-5 * L
    vs = max(1.0, float(np.abs(fw["value"]).max()), float(np.abs(vt).max()))
    np.testing.assert_allclose(J.cpu().numpy(), [r64["J"], r64["l_clip"], r64["l_vf"], r64["l_ent"]], rtol=rt,
                               atol=rt * max(1.0, float(np.abs(adv).max()), vs * vs))
    np.testing.assert_allclose(dlogp.cpu().numpy(), r64["dlogp"], rtol=rt, atol=1e-9)
    np.testing.assert_allclose(dvalue.cpu().numpy(), r64["dvalue"], rtol=1e-5, atol=1e-5 * L * 2 * c1 / state["n_states"])
    np.testing.assert_allclose(dentropy.cpu().numpy(), r64["dentropy"], rtol=1e-5, atol=1e-9)
    # the update chain: gradient of J w.r.t. every weight
    dw = torch.zeros(enc.n_weights, dtype=torch.float32, device="cuda")
    demb = enc.policy_value_backward(batch, emb, dlogp, dvalue, dentropy, dw)
    enc.encode_backward(batch, demb, dw)
    torch.cuda.synchronize()
    bound = O.zero_grads(om)
    _, ref_dw, ref_demb = O.loss_and_grad(om, w, state, r64["dlogp"], r64["dvalue"], r64["dentropy"], bound=bound)
    A, n_near = GC.flip_allowance(om, w, state, ref_demb)
    print(f"undecided ReLU masks in the oracle: {n_near}; largest |logit| {L:.3g}")
    check_grads(dw.cpu().numpy(), ref_dw, O.flatten(om, bound), model, allowance=A, kappa=4e-5 + 1e-5 * L)
    batch.free()
    enc.close()


def test_objective_rejects_invalid_actions(xrl):
    """A recorded action outside its state's slots, or on a masked slot, writes nothing for that
    state and turns J into NaN; the other states' derivatives are those of the valid call."""
    import torch
    model, state = synth.make_config(3, n_states=4, n_cand=6)
    model["precision"] = "fp32"
    state["slot_mask"][np.asarray(state["state_graph_ptr"])[2] + 3] = 0
    w = weights_for(model)
    enc = xrl.Encoder(model, w)
    batch = enc.pack(state)
    pv = enc.policy_value(batch, enc.encode(batch))
    rng = np.random.Generator(np.random.PCG64(5))
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    S = batch.S
    old, adv, vt = (rng.standard_normal(S).astype(np.float32) for _ in range(3))
    good = np.zeros(S, np.int32)
    Jg, dlg, dvg, deg = enc.ppo_objective(batch, pv, t(good), t(old), t(adv), t(vt))
    torch.cuda.synchronize()
    assert torch.isfinite(Jg).all()
    for bad_state, bad_action in ((1, 7), (1, -1), (2, 3)):          # past the last slot, negative, masked
        act = good.copy()
        act[bad_state] = bad_action
        J, dl, dv, de = enc.ppo_objective(batch, pv, t(act), t(old), t(adv), t(vt))
        torch.cuda.synchronize()
        assert torch.isnan(J).all()
        j0, j1 = (int(x) for x in np.asarray(state["state_graph_ptr"])[bad_state:bad_state + 2])
        assert (dl[j0:j1] == 0).all() and dv[bad_state] == 0 and de[bad_state] == 0
        keep = torch.ones(S, dtype=torch.bool, device="cuda")
        keep[bad_state] = False
        assert torch.equal(dv[keep], dvg[keep]) and torch.equal(de[keep], deg[keep])
        gk = torch.ones(batch.G, dtype=torch.bool, device="cuda")
        gk[j0:j1] = False
        assert torch.equal(dl[gk], dlg[gk])
    batch.free()
    enc.close()
