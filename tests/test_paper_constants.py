"""The constants the paper prints (tests/golden/ppo_hyperparameters.txt, each with its citation) are the
defaults of the binding, the workload definitions and the oracle."""
import inspect
import os

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _golden():
    out = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "ppo_hyperparameters.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, value, _cite = line.rstrip("\n").split("\t")
        out[name] = value
    return out


def test_binding_and_oracle_defaults_are_the_papers():
    g = _golden()
    import paper_2403_17031_amd.binding as b
    from oracle import ppo_signals_oracle as O
    sig = inspect.signature(b.ppo_assemble_rewards).parameters
    assert sig["beta"].default == float(g["beta"])
    assert sig["missing_eos_score"].default == float(g["missing_eos_score"])
    sig = inspect.signature(b.ppo_gae).parameters
    assert sig["gamma"].default == float(g["gamma"]) and sig["lam"].default == float(g["lambda"])
    assert inspect.signature(O.assemble_rewards).parameters["missing_eos_score"].default == float(g["missing_eos_score"])
    # epsilon of the printed whiten(): a constant input must come out as exactly 0, and a tiny-variance
    # input must be scaled by 1/sqrt(var + 1e-8), not 1/sqrt(var)
    x = np.array([[0.0, 2e-4]])
    w = O.whiten(x)
    var = x.var()
    np.testing.assert_allclose(w, (x - x.mean()) / np.sqrt(var + float(g["whiten_epsilon"])), rtol=1e-12)
    assert abs(w[0, 1]) < 0.9  # with the epsilon the result is visibly below the +-1 of plain standardisation


def test_workloads_use_the_papers_shapes():
    g = _golden()
    from synth import WORKLOADS
    for i in (2, 3, 4, 5):
        wl = WORKLOADS[i]
        assert wl.temperature == float(g["temperature"])
        assert wl.new_tokens == int(g["response_tokens"])
        assert wl.query_len == int(g["query_tokens"])
        assert wl.model.eos_id == int(g["eos_token_id"])
        assert wl.model.vocab == 50304
    assert WORKLOADS[1].temperature == float(g["temperature"]) and WORKLOADS[1].model.eos_id == 0


def test_value_head_initialisation_scale():
    """Reward Model Details: the scalar head is drawn with standard deviation 1/sqrt(d_model + 1)."""
    from synth import WORKLOADS, make_tensor
    cfg = WORKLOADS[2].model
    v = make_tensor(cfg, 1002, "value_w")
    assert v.shape == (cfg.d_model,)
    assert abs(float(np.std(v)) * np.sqrt(cfg.d_model + 1) - 1.0) < 0.1
