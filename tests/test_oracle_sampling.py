"""Pins for the oracle's sampling path (temperature > 0).

The paper keeps the rejection-sampling scheme of speculative decoding and states that it preserves
the target model's distribution (Sec. 3, last sentence; Related work; App. F reports temperature 1).
S1  inverse-CDF draws: closed forms (uniform weights, one-hot, zero-weight tokens, end points).
S2  distribution preservation, by Monte Carlo over the oracle's own decision functions: the first
    emitted token of a block is distributed as the target's p_0 whatever the draft distribution, and
    given an accepted first token the second is distributed as the target's p_1.
S3  limits: identical draft and target distributions keep every draft token; a target that gives a
    draft token probability 0 always rejects it and never re-draws it; temperature -> 0 turns the
    scheme into the arg-max comparison of the greedy path.
S4  the loop: a draft identical to the target is never rejected; at a vanishing temperature the
    sampled text is the target's greedy text (the zero-temperature invariant of the greedy loop)."""
import math

import numpy as np
import pytest
import torch

from oracle import disco_oracle as O
from workloads import synth as W

F64 = torch.float64


def test_s1_sample_index_closed_forms():
    w = torch.ones(8, dtype=F64)
    for u in (0.0, 0.1, 0.124, 0.126, 0.5, 0.874, 0.876, 0.999999):
        v, margin = O.sample_index(w, u)
        assert v == int(math.floor(u * 8)), u
        assert margin >= 0.0
    # unnormalised weights: same draw as the normalised ones
    assert O.sample_index(5.0 * w, 0.63)[0] == 5
    # one-hot: always that token
    oh = torch.zeros(11, dtype=F64); oh[7] = 3.0
    for u in (0.0, 0.3, 0.99999):
        assert O.sample_index(oh, u)[0] == 7
    # zero-weight tokens are never drawn, also at the ends of the range
    z = torch.tensor([0.0, 0.0, 1.0, 0.0, 3.0, 0.0, 0.0], dtype=F64)
    assert O.sample_index(z, 0.0)[0] == 2
    assert O.sample_index(z, 0.2499)[0] == 2
    assert O.sample_index(z, 0.2501)[0] == 4
    assert O.sample_index(z, 0.9999999)[0] == 4
    # margin: distance to the nearest interval boundary as a fraction of the total
    v, margin = O.sample_index(z, 0.26)
    assert v == 4 and abs(margin - 0.01) < 1e-12
    # softmax at temperature: T = 1 is the plain softmax, T scales the logits
    x = torch.tensor([0.3, -1.0, 2.0], dtype=F64)
    assert torch.allclose(O.softmax_t(x, 1.0), torch.softmax(x, 0), atol=1e-15)
    assert torch.allclose(O.softmax_t(x, 0.5), torch.softmax(2.0 * x, 0), atol=1e-15)


def _random_dist(g, v, zeros=0):
    p = g.random(v) ** 2
    if zeros:
        p[g.choice(v, zeros, replace=False)] = 0.0
    return torch.from_numpy(p / p.sum())


def test_s2_first_and_second_emitted_tokens_follow_the_target():
    g = np.random.default_rng(7)
    V, N = 6, 40000
    q0 = _random_dist(g, V)
    p0 = _random_dist(g, V, zeros=1)                      # the target excludes one token
    q1 = [_random_dist(g, V) for _ in range(V)]           # draft / target rows after first token v
    p1 = [_random_dist(g, V) for _ in range(V)]
    p2 = _random_dist(g, V)
    first = np.zeros(V)
    second = np.zeros((V, V))
    n_second = np.zeros(V)
    us = g.random((N, 5))
    for i in range(N):
        d1, _ = O.sample_index(q0, us[i, 0])
        d2, _ = O.sample_index(q1[d1], us[i, 1])
        n, emit, _ = O.accept_stochastic([0, d1, d2], [q0, q1[d1]], [p0, p1[d1], p2], us[i, 2:4], [us[i, 4]] * 3)
        assert len(emit) == n + 1
        first[emit[0]] += 1
        if n >= 1:
            assert emit[0] == d1
            n_second[d1] += 1
            second[d1, emit[1]] += 1
    sd = np.sqrt(p0.numpy() * (1 - p0.numpy()) / N)
    assert np.all(np.abs(first / N - p0.numpy()) <= 5 * sd + 1e-9), (first / N, p0)
    assert first[np.argmin(p0.numpy())] == 0              # the excluded token is never emitted
    for v in range(V):
        if n_second[v] < 500:
            continue
        pv = p1[v].numpy()
        sdv = np.sqrt(pv * (1 - pv) / n_second[v])
        assert np.all(np.abs(second[v] / n_second[v] - pv) <= 5 * sdv + 1e-9), v
    # acceptance rate of the first draft token = sum_x min(p0, q0)
    acc = sum(n_second) / N
    beta = float(torch.minimum(p0, q0).sum())
    assert abs(acc - beta) < 5 * math.sqrt(beta * (1 - beta) / N)


def test_s3_limits():
    g = np.random.default_rng(3)
    V = 9
    for _ in range(50):
        p = [_random_dist(g, V) for _ in range(4)]
        block = [1] + [int(x) for x in g.integers(0, V, 3)]
        u = g.random(3)
        # identical distributions: min(1, p/q) = 1 > u, everything is kept, the bonus comes from p[3]
        n, emit, _ = O.accept_stochastic(block, p[:3], p, u, [0.4] * 4)
        assert n == 3 and emit[:3] == block[1:] and emit[3] == O.sample_index(p[3], 0.4)[0]
    # a draft token the target excludes is always rejected and cannot come back from the residual
    q = torch.tensor([0.5, 0.5, 0.0], dtype=F64)
    p = torch.tensor([0.0, 0.25, 0.75], dtype=F64)
    for u_a in (0.0, 0.5, 0.999):
        for u_r in (0.0, 0.3, 0.999):
            n, emit, _ = O.accept_stochastic([2, 0], [q], [p, p], [u_a], [u_r, u_r])
            assert n == 0 and emit[0] == 2        # residual max(0, p - q) = [0, 0, 0.75]
    # temperature -> 0: distributions become one-hot at the arg-max and the scheme is the greedy comparison
    for _ in range(30):
        lt = torch.from_numpy(g.normal(size=(5, V)))
        ld = lt[:4] + torch.from_numpy(g.normal(size=(4, V))) * 0.7
        block = [0] + [O.argmax_lowest(ld[j]) for j in range(4)]
        a = [O.argmax_lowest(lt[j]) for j in range(5)]
        n_g, emit_g = O.accept(block, a)
        T = 1e-3
        n_s, emit_s, _ = O.accept_stochastic(block, [O.softmax_t(ld[j], T) for j in range(4)],
                                             [O.softmax_t(lt[j], T) for j in range(5)], g.random(4), g.random(5))
        assert (n_s, emit_s) == (n_g, emit_g)


def _cfg0():
    tw = W.make_weights(W.CFG0_TARGET, seed=0, dtype="f32")
    target = O.Model(W.CFG0_TARGET, tw)
    draft = O.Model(W.CFG0_DRAFT, W.early_exit_draft(tw, 1))
    return tw, target, draft, W.make_classifier(100), W.make_prompt(1, 32, W.CFG0_TARGET.vocab).tolist()


def _uniforms(seed, n):
    return {k: W.make_uniforms(seed, n, k) for k in ("draft", "accept", "resample")}


def test_s4_loop_invariants():
    tw, target, draft, clf, prompt = _cfg0()
    n_new = 24
    u = _uniforms(11, n_new + 16)
    # (a) a draft that is the target itself is never rejected, at any temperature
    same = O.Model(W.CFG0_TARGET, tw)
    r = O.spec_decode_sampling(target, same, clf, prompt, n_new, {"mode": "static", "gamma": 4}, 1.0, u)
    assert all(it["n"] == it["sl"] for it in r["iterations"])
    assert len(r["tokens"]) == n_new
    # (b) at a vanishing temperature every policy emits the target's greedy text
    ref, margins = O.greedy_target(target, prompt, n_new)
    assert min(margins) > 1e-3
    for pol in ({"mode": "static", "gamma": 3}, {"mode": "disco", "tau": 0.55, "sl_max": 6, "pos_mode": "block"}):
        r0 = O.spec_decode_sampling(target, draft, clf, prompt, n_new, pol, 1e-5, u)
        assert r0["tokens"] == ref, pol
    # (c) at temperature 1 the run is a valid schedule: token budget met, cache lengths consistent
    r1 = O.spec_decode_sampling(target, draft, clf, prompt, n_new, {"mode": "disco", "tau": 0.5, "sl_max": 6}, 1.0, u)
    assert len(r1["tokens"]) == n_new
    assert sum(len(it["emit"]) for it in r1["iterations"]) == n_new
    for it in r1["iterations"]:
        assert 0 <= it["n"] <= it["sl"] <= 6 and len(it["emit"]) <= it["n"] + 1
    # same uniforms, same text (the run is a function of its inputs)
    r2 = O.spec_decode_sampling(target, draft, clf, prompt, n_new, {"mode": "disco", "tau": 0.5, "sl_max": 6}, 1.0, u)
    assert r2["tokens"] == r1["tokens"]
