"""Pins for the oracle's search loops (CPU only): hand-worked paths on synthetic loss tables,
closed-form limits (lambda = 1, lambda = 0), local optimality by exhaustive enumeration, and
the paper's qualitative findings under the analytic AI model."""
import itertools

import numpy as np
import pytest

import oracle
import synth
from oracle import search


def _table_callbacks(ai_tab, acc_tab):
    """Separable synthetic model: AI(q) = sum_i ai_tab[i][q_i], AccLoss(q) = sum_i acc_tab[i][q_i]."""
    def ai_fn(q):
        return sum(ai_tab[i][int(b)] for i, b in enumerate(q))

    def accloss_many(schemes):
        return [sum(acc_tab[i][int(b)] for i, b in enumerate(q)) for q in schemes]

    return ai_fn, accloss_many


def test_greedy_hand_worked_two_layers():
    # lambda = 0.5: L = -0.5 AI + 0.5 Acc.  Layer 0: AI 0/4/6, Acc 0/1/9.  Layer 1: AI 0/1/2, Acc 0/3/0.
    # start L = 0.  moves: (0,8): -1.5  (0,4): +1.5  (1,8): +1.0  (1,4): -1.0  -> take (0,8), L = -1.5
    # then: (0,4): dAI 2, dAcc 8 -> +3.0   (1,8): +1.0   (1,4): -1.0 -> take (1,4), L = -2.5 ; L = 2 iterations done
    ai = [{32: 0.0, 8: 4.0, 4: 6.0}, {32: 0.0, 8: 1.0, 4: 2.0}]
    acc = [{32: 0.0, 8: 1.0, 4: 9.0}, {32: 0.0, 8: 3.0, 4: 0.0}]
    q, trace = search.greedy(2, (32, 8, 4), 0.5, *_table_callbacks(ai, acc))
    assert q.tolist() == [8, 4]
    assert [(t["layer"], t["bits"]) for t in trace] == [(-1, 32), (0, 8), (1, 4)]
    assert [t["loss"] for t in trace] == [0.0, -1.5, -2.5]
    # strict reading gives the same path here; with one iteration only the first move is made
    q1, tr1 = search.greedy(2, (32, 8, 4), 0.5, *_table_callbacks(ai, acc), max_iters=1)
    assert q1.tolist() == [8, 32] and len(tr1) == 2


def test_greedy_stops_when_no_move_improves_and_respects_iteration_count():
    ai = [{32: 0.0, 8: 1.0, 4: 2.0}] * 3
    acc = [{32: 0.0, 8: 5.0, 4: 50.0}] * 3
    q, trace = search.greedy(3, (32, 8, 4), 0.5, *_table_callbacks(ai, acc))
    assert q.tolist() == [32, 32, 32] and len(trace) == 1
    # every move helps: 3 iterations = 3 moves, although 6 lowering steps exist (32->8->4 per layer)
    acc0 = [{32: 0.0, 8: 0.0, 4: 0.0}] * 3
    ai2 = [{32: 0.0, 8: 1.0, 4: 1.5}, {32: 0.0, 8: 1.0, 4: 3.0}, {32: 0.0, 8: 0.5, 4: 0.6}]
    q, trace = search.greedy(3, (32, 8, 4), 0.9, *_table_callbacks(ai2, acc0))
    assert [(t["layer"], t["bits"]) for t in trace[1:]] == [(1, 4), (0, 4), (2, 4)]
    # strict reading: a layer that left FP32 is never a candidate again
    ai3 = [{32: 0.0, 8: 2.0, 4: 1.0}, {32: 0.0, 8: 0.1, 4: 0.2}]
    acc3 = [{32: 0.0, 8: 0.0, 4: 0.0}] * 2
    qa, _ = search.greedy(2, (32, 8, 4), 1.0, *_table_callbacks(ai3, acc3), only_fp32_layers=True)
    assert qa.tolist() == [8, 4]


def test_coordinate_descent_hand_worked_and_fixed_point():
    ai = [{32: 0.0, 8: 4.0, 4: 6.0}, {32: 0.0, 8: 1.0, 4: 2.0}]
    acc = [{32: 0.0, 8: 1.0, 4: 9.0}, {32: 0.0, 8: 3.0, 4: 0.0}]
    q, trace = search.coordinate_descent(2, (32, 8, 4), 0.5, *_table_callbacks(ai, acc))
    # layer 0: L(8) = -1.5, L(4) = +1.5 -> 8.  layer 1 (with layer 0 at 8): 8 -> -0.5, 4 -> -2.5 -> 4.  second sweep: nothing
    assert q.tolist() == [8, 4]
    assert [(t["layer"], t["bits"], t["sweep"]) for t in trace[1:]] == [(0, 8, 1), (1, 4, 1)]
    assert trace[-1]["loss"] == -2.5


@pytest.mark.parametrize("seed", range(6))
def test_results_are_local_minima_of_a_non_separable_loss(seed):
    """Random loss over 3 layers x {32, 8, 4} with interactions; every accepted greedy step is the
    best single-layer lowering, and coordinate descent ends where no single-layer change helps."""
    rng = np.random.Generator(np.random.PCG64(seed))
    Q = (32, 8, 4)
    table = {q: float(rng.normal()) for q in itertools.product(Q, repeat=3)}
    table[(32, 32, 32)] = 0.5

    def ai_fn(q):
        return 0.0

    def accloss_many(schemes):
        return [table[tuple(int(b) for b in q)] for q in schemes]

    q, trace = search.coordinate_descent(3, Q, 0.0, ai_fn, accloss_many)
    here = table[tuple(q.tolist())]
    for i in range(3):
        for b in Q:
            n = q.copy()
            n[i] = b
            assert table[tuple(n.tolist())] >= here
    g, gtrace = search.greedy(3, Q, 0.0, ai_fn, accloss_many)
    cur = [32, 32, 32]
    for step in gtrace[1:]:
        lower = {}
        for i in range(3):
            for b in Q:
                if b < cur[i]:
                    n = list(cur)
                    n[i] = b
                    lower[(i, b)] = table[tuple(n)]
        best = min(lower.values())
        assert step["loss"] == best and best < table[tuple(cur)]
        cur[step["layer"]] = step["bits"]
    assert cur == g.tolist()
    assert len(gtrace) <= 4


def test_limits_on_resnet20_with_the_analytic_ai_model():
    """lambda = 1 (loss = -AI): AI rises with every lowering, so greedy sends one layer per iteration
    straight to the lowest width, widest layers first, and ends all-INT4 after L iterations;
    lambda = 0 with a non-negative accuracy loss never leaves FP32."""
    nodes = synth.resnet_cifar(3)
    desc = synth.desc_array(nodes)

    def ai_fn(q):
        return oracle.layer_ai(desc, q)[2]

    def no_acc_loss(schemes):
        return [0.0 for _ in schemes]

    q, trace = search.greedy(20, (32, 8, 4), 1.0, ai_fn, no_acc_loss)
    assert q.tolist() == [4] * 20
    assert all(t["bits"] == 4 for t in trace[1:])
    order = [t["layer"] for t in trace[1:]]
    n_weights = [int(d[1]) * int(d[2]) * (9 if d[0] == 0 else 1) for d in desc if d[12] >= 0]
    picked = [n_weights[i] for i in order]
    assert picked == sorted(picked, reverse=True)
    # the paper's Table 1 shows final widths of 32 or 4 only at lambda = 0.9: with a per-layer accuracy
    # cost that is the same for 8 and 4 bits the analytic AI term always prefers 4 over 8
    def flat_cost(schemes):
        return [0.02 * sum(int(b) != 32 for b in s) for s in schemes]

    q9, _ = search.coordinate_descent(20, (32, 8, 4), 0.9, ai_fn, flat_cost)
    assert set(q9.tolist()) <= {32, 4}
    q0, t0 = search.greedy(20, (32, 8, 4), 0.0, ai_fn, flat_cost)
    assert q0.tolist() == [32] * 20 and len(t0) == 1


def test_search_on_the_oracle_forward_pass_is_consistent():
    wl = synth.make_workload(0, n_images=24)
    ai_fn, accloss_many = search.model_callbacks(wl["desc"], wl["weights"], wl["biases"], wl["images"])
    q, trace = search.greedy(wl["L"], (32, 8, 4), 0.9, ai_fn, accloss_many, max_iters=3)
    assert len(trace) >= 2 and all(b in (32, 8, 4) for b in q.tolist())
    final = search.loss(0.9, ai_fn(q), accloss_many([q])[0])
    assert final == pytest.approx(trace[-1]["loss"], rel=1e-12)
    losses = [t["loss"] for t in trace]
    assert all(b < a for a, b in zip(losses, losses[1:]))
