"""Pins for the policy-gradient oracle (CPU only): the rows the paper prints in Figure 6 (Sigmoid
model) and Figure 9 (Softmax model), closed forms and library forms of the discount recurrence,
a brute force, invariants of the softmax gradient, and planted mistakes the pins must catch."""
import json
import math
import os
import subprocess

import numpy as np
import pytest

from oracle import policy_gradient as pgo
from oracle.policy_gradient import PgOracleLib

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "pg_oracle.c")
FIG6 = json.load(open(os.path.join(HERE, "golden", "pg_figure6.json")))
FIG9 = json.load(open(os.path.join(HERE, "golden", "pg_figure9.json")))


def check_figure6(lib):
    rows = np.array(FIG6["rows"], dtype=np.float64)
    aprob, action, dlogps, diff, old_w, new_w, data, old_res, new_res = rows.T
    np.testing.assert_array_equal(lib.sigmoid_sample_action(aprob, np.full(4, 0.5)), action.astype(np.int64))
    d = lib.sigmoid_dlogps(aprob, action.astype(np.int64))
    np.testing.assert_allclose(d, dlogps, rtol=0, atol=1e-15)
    bd = lib.bottom_diff(d, None, True)            # reward weight 1, as in the figure
    np.testing.assert_allclose(bd, diff, rtol=0, atol=1e-15)
    # the rest of the printed row follows from the diff: the solver subtracts it
    np.testing.assert_allclose(old_w - bd, new_w, rtol=0, atol=1e-15)
    np.testing.assert_allclose(old_w * data, old_res, rtol=0, atol=1e-15)
    np.testing.assert_allclose((old_w - bd) * data, new_res, rtol=0, atol=1e-15)


def check_figure9(lib):
    for row in FIG9["rows"]:
        probs = np.array(row["probs"])
        logits = np.array([[math.log(p) if p > 0 else -math.inf for p in probs]])
        action = [int(np.argmax(row["targets"]))]
        p, d = lib.softmax_dlogps(logits, action)
        np.testing.assert_allclose(p[0], probs, rtol=0, atol=1e-15)
        np.testing.assert_allclose(d[0], row["gradient"], rtol=0, atol=1e-15)
        bd = lib.bottom_diff(d, None, False)[0]
        np.testing.assert_allclose(bd, row["diff"], rtol=0, atol=1e-15)
        new_w = row["old_weight"] - bd
        np.testing.assert_allclose(new_w, row["new_weight"], rtol=0, atol=1e-15)
        np.testing.assert_allclose(row["old_weight"] * np.array(row["data"]), row["old_result"], rtol=0, atol=1e-15)
        np.testing.assert_allclose(new_w * np.array(row["data"]), row["new_result"], rtol=0, atol=1e-15)


def check_discount(lib):
    r = np.random.default_rng(3)
    lengths = [0, 1, 2, 7, 64, 65, 130, 0, 3]
    offsets = np.concatenate([[0], np.cumsum(lengths)])
    reward = r.standard_normal(offsets[-1])
    for gamma in (0.0, 0.5, 0.99, 1.0):
        got = lib.discount_rewards(reward, offsets, gamma)
        want = np.zeros_like(reward)
        for e in range(len(lengths)):                      # brute force: the sum written out
            for t in range(offsets[e], offsets[e + 1]):
                want[t] = sum(gamma ** (s - t) * reward[s] for s in range(t, offsets[e + 1]))
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # closed form: constant reward 1 over T steps -> (1 - gamma^(T-t)) / (1 - gamma)
    T, gamma = 200, 0.97
    got = lib.discount_rewards(np.ones(T), [0, T], gamma)
    np.testing.assert_allclose(got, (1 - gamma ** (T - np.arange(T))) / (1 - gamma), rtol=1e-12)
    # gamma = 1 is a suffix sum (numpy), gamma = 0 the reward itself
    x = r.standard_normal(50)
    np.testing.assert_allclose(lib.discount_rewards(x, [0, 50], 1.0), np.cumsum(x[::-1])[::-1], rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(lib.discount_rewards(x, [0, 20, 50], 0.0), x)
    # modulation: one weight per step, every action of the step
    d = r.standard_normal((6, 3))
    w = r.standard_normal(6)
    np.testing.assert_allclose(lib.bottom_diff(d, w, False), d * w[:, None], rtol=1e-15)
    np.testing.assert_allclose(lib.bottom_diff(d[:, 0].copy(), w, True), -d[:, 0] * w, rtol=1e-15)


def _suite(lib):
    check_figure6(lib)
    check_figure9(lib)
    check_discount(lib)


def test_figure6_sigmoid_rows():
    check_figure6(pgo._load())


def test_figure9_softmax_rows():
    check_figure9(pgo._load())


def test_discount_brute_force_and_closed_forms():
    check_discount(pgo._load())


def test_sample_action_threshold():
    # random < Aprob picks action 0; equality picks 1
    np.testing.assert_array_equal(pgo.sigmoid_sample_action([0.3, 0.3, 0.3, 0.0, 1.0], [0.29, 0.3, 0.31, 0.0, 0.999]),
                                  [0, 1, 1, 1, 0])


def test_softmax_gradient_invariants():
    r = np.random.default_rng(5)
    logits = r.standard_normal((40, 7)) * 3
    action = r.integers(0, 7, 40)
    p, d = pgo.softmax_dlogps(logits, action)
    np.testing.assert_allclose(p.sum(1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(d.sum(1), 0.0, atol=1e-14)
    # shifting a row's logits changes nothing; huge logits do not overflow
    p2, d2 = pgo.softmax_dlogps(logits + 1000.0, action)
    np.testing.assert_allclose(p2, p, rtol=1e-10)
    # gradient of -log softmax[action] by central differences
    eps = 1e-6
    for t in range(0, 40, 7):
        for a in range(7):
            hi, lo = logits[t].copy(), logits[t].copy()
            hi[a] += eps
            lo[a] -= eps
            f = lambda l: -(l[action[t]] - np.log(np.exp(l).sum()))
            assert abs((f(hi) - f(lo)) / (2 * eps) - d[t, a]) < 1e-8
    # two actions: Dlogps of the Sigmoid model is minus the Softmax gradient of action 0's logit
    ap = p[:, 0] / (p[:, 0] + p[:, 1])
    two = np.log(np.stack([ap, 1 - ap], 1))
    act = (action % 2)
    _, d_two = pgo.softmax_dlogps(two, act)
    np.testing.assert_allclose(pgo.sigmoid_dlogps(ap, act), -d_two[:, 0], rtol=1e-12, atol=1e-14)


def test_argument_checks():
    with pytest.raises(ValueError):
        pgo.sigmoid_dlogps([0.5], [2])
    with pytest.raises(ValueError):
        pgo.softmax_dlogps(np.zeros((2, 3)), [0, 3])
    with pytest.raises(ValueError):
        pgo.discount_rewards(np.zeros(4), [0, 3, 2, 4], 0.9)
    with pytest.raises(ValueError):
        pgo.discount_rewards(np.zeros(4), [1, 4], 0.9)
    assert pgo.discount_rewards(np.zeros(0), [0], 0.9).size == 0
    assert pgo.sigmoid_dlogps([], []).size == 0


MUTANTS = [
    ("sample_inverted", "action[t] = (random[t] < aprob[t]) ? 0 : 1;", "action[t] = (random[t] < aprob[t]) ? 1 : 0;"),
    ("dlogps_branches_swapped", "(action[t] == 0) ? 1.0 - aprob[t] : 0.0 - aprob[t];",
     "(action[t] == 1) ? 1.0 - aprob[t] : 0.0 - aprob[t];"),
    ("dlogps_plus", "(action[t] == 0) ? 1.0 - aprob[t] : 0.0 - aprob[t];", "(action[t] == 0) ? 1.0 - aprob[t] : 0.0 + aprob[t];"),
    ("softmax_target_minus_softmax", "dlogps[t * actions + a] = softmax - target;", "dlogps[t * actions + a] = target - softmax;"),
    ("softmax_no_normalisation", "const double softmax = exp(l[a] - top) / sum;", "const double softmax = exp(l[a] - top);"),
    ("softmax_target_wrong_action", "const double target = (a == action[t]) ? 1.0 : 0.0;",
     "const double target = (a != action[t]) ? 1.0 : 0.0;"),
    ("sigmoid_sign_of_diff", "const double sign = sigmoid_model ? -1.0 : 1.0;", "const double sign = 1.0;"),
    ("softmax_sign_of_diff", "const double sign = sigmoid_model ? -1.0 : 1.0;", "const double sign = -1.0;"),
    ("discount_forward_in_time", "for (int64_t t = offsets[e + 1] - 1; t >= offsets[e]; --t) {\n      running = reward[t] + gamma * running;\n      discounted[t] = running;",
     "for (int64_t t = offsets[e]; t < offsets[e + 1]; ++t) {\n      running = reward[t] + gamma * running;\n      discounted[t] = running;"),
    ("discount_crosses_episodes", "double running = 0.0; /* R past the end of the episode */\n    for", "double running = (e + 1 < episodes && offsets[e + 1] < offsets[episodes]) ? discounted[offsets[e + 1]] : 0.0;\n    for"),
    ("discount_scales_reward", "running = reward[t] + gamma * running;", "running = gamma * (reward[t] + running);"),
    ("modulation_ignores_reward", "(discounted ? discounted[t] : 1.0)", "1.0"),
]


def _build(text, out_dir, name):
    c, so = os.path.join(out_dir, name + ".c"), os.path.join(out_dir, name + ".so")
    with open(c, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-I", os.path.dirname(SRC), "-o", so, c, "-lm"], check=True)
    return PgOracleLib(so)


def test_unmodified_source_passes_the_suite(tmp_path):
    _suite(_build(open(SRC).read(), str(tmp_path), "clean"))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    src = open(SRC).read()
    assert old in src, f"mutation site for {name} not found"
    lib = _build(src.replace(old, new), str(tmp_path), name)
    with pytest.raises((AssertionError, ValueError)):
        _suite(lib)
