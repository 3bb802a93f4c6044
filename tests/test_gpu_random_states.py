"""Robustness sweep: unstructured random states (empty graphs, self loops, repeated edges, edges in
any direction, random masks) through encode + heads against the oracle, in every mode, on both the
one-launch encoder (small graphs) and the streaming / persistent kernels. Tolerances as in
test_gpu_forward.py."""
import numpy as np
import pytest

import synth
from test_gpu_forward import run_case, weights_for

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xrl():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2304_14698_amd as x
    x.load_library()
    return x


@pytest.mark.parametrize("hidden,precision", [(64, "fp32"), (128, "fp32"), (64, "bf16"), (128, "bf16"), (256, "bf16")])
def test_random_states(xrl, hidden, precision, monkeypatch):
    model, _ = synth.make_config(1)
    model.update(hidden=hidden, precision=precision, rounds=2)
    rng = np.random.Generator(np.random.PCG64(2024))
    w = weights_for(model)
    for k in range(6):
        # small graphs (one-launch encoder where the mode has it), then larger ones; the last two
        # with the persistent kernels forced onto a few hundred rows
        big = k >= 2
        monkeypatch.setenv("XRL_PERSISTENT_MIN_ROWS", "0" if k >= 4 else "8192")
        state = synth.random_states(rng, model, n_states=int(rng.integers(1, 5)), max_graphs=5,
                                    max_nodes=400 if big else 100, edge_factor=(0.0, 1.5))
        run_case(xrl, model, state, w, check_inter=True)


@pytest.mark.parametrize("hidden", [64, 128])
def test_random_states_backward_fp32(xrl, hidden):
    """The same kind of states through the whole backward (heads + encoder) against the oracle's
    reverse mode, fp32 (elementwise criterion of test_gpu_backward.py)."""
    from test_gpu_backward import run_backward_case
    model, _ = synth.make_config(1)
    model.update(hidden=hidden, precision="fp32", rounds=2)
    rng = np.random.Generator(np.random.PCG64(77))
    w = weights_for(model)
    for k in range(4):
        state = synth.random_states(rng, model, n_states=int(rng.integers(1, 4)), max_graphs=4,
                                    max_nodes=300 if k >= 2 else 90, edge_factor=(0.0, 1.5))
        run_backward_case(xrl, model, state, w, seed=5 + k)
