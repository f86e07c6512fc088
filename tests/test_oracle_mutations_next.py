"""Do the pins of the later oracles have teeth?  One plausible mistake at a time is planted in a
*copy* of an oracle module (policy gradient, REINFORCE accumulation, the simulator's memory
model), the copy is loaded in place of the module the pins use, and at least one pin must fail.
CPU only."""
import importlib.util
import os
import sys

import pytest

import oracle
import test_oracle_gradient as pins_gradient
import test_oracle_reinforce as pins_reinforce
import test_oracle_simulator as pins_simulator

HERE = os.path.dirname(oracle.__file__)


def load_mutant(filename, old, new, tmp_path):
    text = open(os.path.join(HERE, filename)).read()
    assert text.count(old) == 1, f"mutation anchor not unique: {old!r}"
    path = tmp_path / filename
    path.write_text(text.replace(old, new))
    name = "oracle._mutant_" + filename[:-3]
    spec = importlib.util.spec_from_file_location(name, str(path))
    mod = importlib.util.module_from_spec(spec)
    mod.__package__ = "oracle"                 # the copies keep their relative imports
    sys.modules[name] = mod
    try:
        spec.loader.exec_module(mod)
    finally:
        sys.modules.pop(name, None)
    return mod


def some_pin_fails(pins):
    for pin in pins:
        try:
            pin()
        except Exception:                        # an assertion, or the mutant breaks outright
            return True
    return False


GRADIENT = [
    ("ReLU missing in the embedding networks", "x = torch.relu(x @ W + b)", "x = x @ W + b"),
    ("residual self term dropped", "s[v] = s[v] + _mlp(par, g_name, n_layers, agg)", "s[v] = _mlp(par, g_name, n_layers, agg)"),
    ("f and g swapped in the top-down sweep", '_sweep(par, "f_td", "g_td"', '_sweep(par, "g_td", "f_td"'),
    ("messages are the raw states", "msg[v] = _mlp(par, f_name, n_layers, s[v])", "msg[v] = s[v]"),
    ("log-probability without the normaliser", "lp = torch.log_softmax(logits, dim=0)[int(actions[b])]", "lp = logits[int(actions[b])]"),
    ("scalar of the state ignored", "grad += float(coeff[b]) * g.numpy()", "grad += g.numpy()"),
    ("ancestors and descendants swapped", "cls = 0 if u in up else (1 if u in down else 2)", "cls = 1 if u in up else (0 if u in down else 2)"),
    ("pooling ignores the device", "d = int(placement[u]) if group_by_device else 0", "d = 0"),
    ("policy hidden layer linear", "return torch.relu(z @ W1 + b1) @ W2 + b2", "return (z @ W1 + b1) @ W2 + b2"),
    ("is-current and is-visited swapped", "phi[cur, 2 + D] = 1.0\n    phi[:, 3 + D] = feats[:, 2]", "phi[cur, 3 + D] = 1.0\n    phi[:, 2 + D] = feats[:, 2]"),
]


@pytest.mark.parametrize("what,old,new", GRADIENT, ids=[m[0] for m in GRADIENT])
def test_gradient_oracle_mistake_is_caught(what, old, new, tmp_path, monkeypatch):
    monkeypatch.setattr(pins_gradient, "og", load_mutant("gradient.py", old, new, tmp_path))
    pins = [lambda: pins_gradient.test_forward_equals_the_c_oracle(2, 1, 1),
            lambda: pins_gradient.test_gradient_equals_central_differences_of_the_c_oracle(2, 1, 1),
            pins_gradient.test_output_bias_gradient_is_onehot_minus_pi,
            pins_gradient.test_linear_in_coeff_and_additive_over_the_batch]
    assert some_pin_fails(pins), f"no pin notices: {what}"


REINFORCE = [
    ("return excludes the step's own reward", "for u in range(t, r.shape[0]):", "for u in range(t + 1, r.shape[0]):"),
    ("baseline is the sum, not the mean", "base[:, g] = G[:, members].sum(axis=1) / len(members)", "base[:, g] = G[:, members].sum(axis=1)"),
    ("baseline added instead of subtracted", "coeff[:, b] -= base[:, group[b]]", "coeff[:, b] += base[:, group[b]]"),
    ("baseline of step 0 used for every step", "coeff[:, b] -= base[:, group[b]]", "coeff[:, b] -= base[0, group[b]]"),
]


@pytest.mark.parametrize("what,old,new", REINFORCE, ids=[m[0] for m in REINFORCE])
def test_reinforce_oracle_mistake_is_caught(what, old, new, tmp_path, monkeypatch):
    monkeypatch.setattr(pins_reinforce, "orf", load_mutant("reinforce.py", old, new, tmp_path))
    pins = [pins_reinforce.test_returns_of_constant_and_single_rewards,
            pins_reinforce.test_returns_equal_reversed_cumulative_sum,
            pins_reinforce.test_baseline_is_the_group_mean_and_advantages_cancel,
            pins_reinforce.test_better_rollout_gets_positive_weight]
    assert some_pin_fails(pins), f"no pin notices: {what}"


MEMORY = [
    ("an output is freed when its op ends, consumers ignored",
     "free[v, d] = max(float(op_end[v]), last_use[v, d])", "free[v, d] = float(op_end[v])"),
    ("closed intervals: what is freed at t still counts at t", "(a <= t) & (t < f)", "(a <= t) & (t <= f)"),
    ("a remote copy exists from the producer's start", "alloc[v, o] = float(arrival[v, o])", "alloc[v, o] = float(op_start[v])"),
    ("the source does not wait for its transfer",
     "free[v, d] = max(free[v, d], float(arrival_last[v, o]))   # the source stays until it has been sent", "pass"),
    ("with repeated crossings the source waits for the first arrival only",
     "arrival, arrival_last = arrival if isinstance(arrival, tuple) else (arrival, arrival)",
     "arrival, arrival_last = (arrival[0], arrival[0]) if isinstance(arrival, tuple) else (arrival, arrival)"),
    ("with repeated crossings the copy appears at the last arrival",
     "arrival, arrival_last = arrival if isinstance(arrival, tuple) else (arrival, arrival)",
     "arrival, arrival_last = (arrival[1], arrival[1]) if isinstance(arrival, tuple) else (arrival, arrival)"),
    ("per-child transfers still release every child waiting on the device",
     "for c in ([child] if per_child else children[o]):", "for c in children[o]:"),
    ("per-child transfers are sent once per device after all",
     "elif per_child:", "elif per_child and pc not in sent:\n                    sent.add(pc)"),
    ("an output is allocated when its op ends", "alloc[v, d] = float(op_start[v])", "alloc[v, d] = float(op_end[v])"),
    ("the penalty ignores the limit", "float(r) + c * (float(m) - float(M))", "float(r) + c * float(m)"),
    ("last consumer taken over all devices", "last_use[u, pc] = max(last_use[u, pc], float(op_end[c]))",
     "last_use[u, :] = np.maximum(last_use[u, :], float(op_end[c]))"),
]


@pytest.mark.parametrize("what,old,new", MEMORY, ids=[m[0] for m in MEMORY])
def test_memory_model_mistake_is_caught(what, old, new, tmp_path, monkeypatch):
    monkeypatch.setattr(pins_simulator, "sim", load_mutant("simulator.py", old, new, tmp_path))
    pins = [pins_simulator.test_peak_memory_of_a_chain_on_one_device,
            pins_simulator.test_peak_memory_with_a_transfer,
            pins_simulator.test_peak_memory_fork_join_and_bounds,
            pins_simulator.test_penalised_runtime_formula,
            pins_simulator.test_two_children_on_one_remote_device_one_transfer_or_two,
            pins_simulator.test_per_child_transfers_on_a_mixed_fan_out]
    assert some_pin_fails(pins), f"no pin notices: {what}"
