"""The hyper-parameters the paper prints (Appendix E, Table 2; copied into tests/golden/ with
their citation) are the defaults of the synthetic workloads."""
import os

from paper_2502_20190_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    return [l.split() for l in open(os.path.join(GOLDEN, name)) if l.strip() and not l.startswith("#")]


def test_dqn_columns():
    table = {}
    for col, key, value in _rows("table2_dqn_hyperparameters.txt"):
        table.setdefault(col, {})[key] = float(value)
    for cfg, col in (("c2", "cartpole"), ("c3", "cartpole"), ("c4", "atari"), ("c5", "atari")):
        wl, t = synth.WORKLOADS[cfg], table[col]
        assert wl.gamma == t["gamma"] and wl.eps == t["adam_eps"]
        assert wl.lr == t["learning_rate"] and wl.target_interval == t["target_update_interval"]
    # config 1 takes its learning rate from the workload list, the rest from the CartPole column
    c1 = synth.WORKLOADS["c1"]
    assert c1.gamma == table["cartpole"]["gamma"] and c1.eps == table["cartpole"]["adam_eps"]


def test_ppo_column():
    t = {k: float(v) for k, v in _rows("table2_ppo_hyperparameters.txt")}
    h = synth.PPO_HYPER
    assert h["gamma"] == t["gamma"] and h["lam"] == t["gae"]
    assert h["lr"] == t["learning_rate"] and h["eps"] == t["adam_eps"]
    _, _, hidden, _, _, rollout, _ = synth.PPO_WORKLOADS["p1"]
    assert set(hidden) == {int(t["hidden_layer"])} and rollout == int(t["rollout_length"])
    assert synth.PPO_WORKLOADS["p2"][5] == int(t["rollout_length"])
