"""Oracle of the AIQ search loops (TEST INFRASTRUCTURE ONLY, plain Python).

Follows the paper's Approach section:
  loss      L(q; lambda) = -lambda * AI(q) + (1 - lambda) * AccLoss(q)            [Problem Formulation]
  greedy    start all-FP32; per iteration evaluate every move "lower layer i to b in Q",
            take the move with the smallest Delta L if it is negative; as many iterations
            as layers                                                              [Search, Greedy search]
  coordinate descent
            start all-FP32; for each layer in turn pick argmin_b L with the others fixed;
            repeat passes until a pass changes nothing                             [Search, Coordinate descent]

Readings where the paper is silent: AccLoss is in percentage points (100 * (1 - accuracy));
a greedy move may lower any layer that still has a lower width in Q (strict reading
`only_fp32_layers`: a layer moves once, from FP32); when no move improves the loss the
greedy search stops (later iterations would see the same candidates); ties go to the first
candidate in (layer ascending, width descending) order, and coordinate descent keeps the
current width unless another is strictly better.

ai_fn(scheme) -> float and accloss_many(list of schemes) -> list of float are supplied by
the caller, so the loops can be pinned on synthetic tables as well as run on the oracle's
forward pass.
"""
from __future__ import annotations

import numpy as np


def loss(lam, ai, acc_loss):
    return -lam * ai + (1.0 - lam) * acc_loss


def greedy(L, Q, lam, ai_fn, accloss_many, max_iters=None, only_fp32_layers=False):
    """Returns (scheme uint8[L], trace); trace[0] is the start, each later entry one accepted move."""
    Q = sorted(int(b) for b in Q)[::-1]
    q = np.full(L, Q[0], dtype=np.uint8)
    cur = loss(lam, ai_fn(q), accloss_many([q])[0])
    trace = [dict(layer=-1, bits=int(Q[0]), loss=cur)]
    for _ in range(L if max_iters is None else max_iters):
        moves = []
        for i in range(L):
            if only_fp32_layers and q[i] != Q[0]:
                continue
            for b in Q:
                if b < q[i]:
                    moves.append((i, b))
        if not moves:
            break
        cands = []
        for i, b in moves:
            c = q.copy()
            c[i] = b
            cands.append(c)
        acc = accloss_many(cands)
        deltas = [loss(lam, ai_fn(c), a) - cur for c, a in zip(cands, acc)]
        k = int(np.argmin(deltas))  # first minimum
        if not deltas[k] < 0:
            break
        q = cands[k]
        cur = cur + deltas[k]
        trace.append(dict(layer=moves[k][0], bits=moves[k][1], loss=cur))
    return q, trace


def coordinate_descent(L, Q, lam, ai_fn, accloss_many, max_passes=50):
    """Returns (scheme uint8[L], trace); one trace entry per accepted per-layer update."""
    Q = sorted(int(b) for b in Q)[::-1]
    q = np.full(L, Q[0], dtype=np.uint8)
    cur = loss(lam, ai_fn(q), accloss_many([q])[0])
    trace = [dict(layer=-1, bits=int(Q[0]), loss=cur, sweep=0)]
    for sweep in range(1, max_passes + 1):
        updated = False
        for i in range(L):
            others = [b for b in Q if b != q[i]]
            cands = []
            for b in others:
                c = q.copy()
                c[i] = b
                cands.append(c)
            acc = accloss_many(cands)
            vals = [loss(lam, ai_fn(c), a) for c, a in zip(cands, acc)]
            k = int(np.argmin(vals))
            if vals[k] < cur:
                q, cur, updated = cands[k], vals[k], True
                trace.append(dict(layer=i, bits=others[k], loss=cur, sweep=sweep))
        if not updated:
            break
    return q, trace


def model_callbacks(desc, weights, biases, images):
    """ai_fn / accloss_many backed by the oracle's own AI model and forward pass."""
    import oracle
    n = images.shape[0]

    def ai_fn(q):
        return oracle.layer_ai(desc, q)[2]

    def accloss_many(schemes):
        r = oracle.eval_schemes(desc, weights, biases, images, np.stack(schemes), want_logits=False)
        return [100.0 * (1.0 - a / n) for a in r["agree"]]

    return ai_fn, accloss_many
