"""Pins for the oracle's classifier-training path (Sec. 4 "SL classifier training", App. D.1 / D.2).

T1  the gradient step: one epoch of clf_train equals one step of torch.autograd on the same loss
    (library routine), and the loss it reports equals F.binary_cross_entropy on the sigmoid output.
T2  folding: the returned parameters applied to RAW features give the score of the trained
    parameters applied to standardised features.
T3  behaviour: the loss falls monotonically for a small step; a linearly separable toy set reaches
    F1 = 1; F1 and the confusion counts against hand-counted cases.
T4  labelling run: its labels are the match vector that fixes every policy's schedule (the same
    vector the loop tests derive from App. D.1), its features those of the loop's first draft step."""
import math

import pytest
import torch
import torch.nn.functional as F

from oracle import disco_oracle as O
from workloads import synth as W

F64 = torch.float64


def _data(n=300, seed=0, hidden=16):
    g = torch.Generator().manual_seed(seed)
    feats = torch.rand(n, 12, generator=g, dtype=F64)
    feats[:, 11] = torch.arange(1, n + 1, dtype=F64)            # a large-scale component, like the position
    y = ((feats[:, 0] + 0.3 * feats[:, 10]) > 0.7).to(torch.int32)
    init = {"W1": torch.randn(hidden, 12, generator=g, dtype=F64) * 0.1, "b1": torch.randn(hidden, generator=g, dtype=F64) * 0.1,
            "w2": torch.randn(hidden, generator=g, dtype=F64) * 0.1, "b2": torch.randn(1, generator=g, dtype=F64) * 0.1}
    return feats, y, init


def test_t1_one_epoch_is_one_autograd_step():
    feats, y, init = _data()
    lr = 0.3
    # reference: autograd on the same loss in the standardised space
    mu = feats.mean(0); sd = feats.std(0, unbiased=False).clamp(min=1e-6)
    s = (feats - mu) / sd
    p = {k: v.clone().requires_grad_(True) for k, v in init.items()}
    z = torch.relu(s @ p["W1"].T + p["b1"]) @ p["w2"] + p["b2"][0]
    loss = F.binary_cross_entropy(torch.sigmoid(z), y.to(F64))
    loss.backward()
    want = {k: (v - lr * v.grad).detach() for k, v in p.items()}
    got, losses = O.clf_train(feats, y, init, 1, lr)
    assert abs(losses[0] - float(loss.detach())) < 1e-12
    # unfold the oracle's result and compare in the standardised space
    W1 = got["W1"].to(F64) * sd
    b1 = got["b1"].to(F64) + (W1 * (mu / sd)).sum(1)
    assert torch.allclose(W1, want["W1"], atol=1e-6) and torch.allclose(b1, want["b1"], atol=1e-6)
    assert torch.allclose(got["w2"].to(F64), want["w2"], atol=1e-6) and torch.allclose(got["b2"].to(F64), want["b2"], atol=1e-6)


def test_t2_folded_parameters_consume_raw_features():
    feats, y, init = _data(n=120, seed=3)
    got, _ = O.clf_train(feats, y, init, 40, 0.5)
    # retrain by hand in the standardised space with autograd-free recursion = the same function; compare scores
    mu = feats.mean(0); sd = feats.std(0, unbiased=False).clamp(min=1e-6)
    W1 = got["W1"].to(F64) * sd
    b1 = got["b1"].to(F64) + (W1 * (mu / sd)).sum(1)
    for i in (0, 7, 55, 119):
        s = (feats[i] - mu) / sd
        z = torch.relu(W1 @ s + b1) @ got["w2"].to(F64) + got["b2"].to(F64)[0]
        c_std = 1.0 / (1.0 + math.exp(-float(z)))
        c_raw = O.classifier(feats[i].to(torch.float32), got)
        assert abs(c_std - c_raw) < 2e-5          # float32 rounding of the folded parameters and of the features


def test_t3_training_behaviour_and_f1():
    feats, y, init = _data(n=400, seed=1)
    clf, losses = O.clf_train(feats, y, init, 300, 0.5)
    assert all(b <= a + 1e-12 for a, b in zip(losses, losses[1:]))
    assert losses[-1] < 0.5 * losses[0]
    ev = O.clf_eval(feats.to(torch.float32), y, clf, 0.5)
    assert ev["f1"] > 0.9
    # separable toy set: one informative component
    g = torch.Generator().manual_seed(5)
    f2 = torch.rand(200, 12, generator=g, dtype=F64)
    y2 = (f2[:, 3] > 0.5).to(torch.int32)
    f2[:, 3] += torch.where(y2 > 0, 0.2, -0.2)
    clf2, _ = O.clf_train(f2, y2, init, 2000, 1.0)
    assert O.clf_eval(f2.to(torch.float32), y2, clf2, 0.5)["f1"] == 1.0
    # confusion counts by hand: zero weights give C = 0.5 everywhere
    zero = {"W1": torch.zeros(4, 12), "b1": torch.zeros(4), "w2": torch.zeros(4), "b2": torch.zeros(1)}
    lab = torch.tensor([1, 1, 0, 1, 0], dtype=torch.int32)
    ev = O.clf_eval(torch.zeros(5, 12), lab, zero, 0.5)          # C = 0.5 >= tau: everything predicted accepted
    assert (ev["tp"], ev["fp"], ev["fn"], ev["tn"]) == (3, 2, 0, 0) and abs(ev["f1"] - 6 / 8) < 1e-12
    ev = O.clf_eval(torch.zeros(5, 12), lab, zero, 0.51)         # nothing predicted accepted
    assert (ev["tp"], ev["fp"], ev["fn"], ev["tn"]) == (0, 0, 3, 2) and ev["f1"] == 0.0


def test_t4_labelling_run_is_the_match_vector():
    tw = W.make_weights(W.CFG0_TARGET, seed=0, dtype="f32")
    target = O.Model(W.CFG0_TARGET, tw)
    draft = O.Model(W.CFG0_DRAFT, W.early_exit_draft(tw, 1))
    clf = W.make_classifier(100)
    prompt = W.make_prompt(1, 32, W.CFG0_TARGET.vocab).tolist()
    n_new = 40
    ref, _ = O.greedy_target(target, prompt, n_new)
    force = {"mask": W.make_force_mask(5, n_new, 0.6), "tokens": ref}
    run = O.label_run(draft, prompt, ref, force)
    assert run["feats"].shape == (n_new, 12) and run["labels"].shape == (n_new,)
    assert all(int(run["labels"][p]) == 1 for p in range(n_new) if bool(force["mask"][p]))      # forced positions match
    assert 0 < int(run["labels"].sum()) < n_new
    assert [float(run["feats"][p, 11]) for p in range(n_new)] == [float(p + 1) for p in range(n_new)]
    # the accepted counts of a static-lookahead run are the run lengths of ones in this vector
    r = O.spec_decode(target, draft, clf, prompt, n_new, {"mode": "static", "gamma": 4}, force=force)
    pos = 0
    for it in r["iterations"]:
        run_len = 0
        while run_len < it["sl"] and int(run["labels"][pos + run_len]) == 1:
            run_len += 1
        assert it["n"] == run_len
        # the first draft step of the iteration sees exactly the labelling run's context
        if it["steps"]:
            assert torch.allclose(it["steps"][0]["feats"][:11], run["feats"][pos][:11], rtol=1e-6, atol=1e-9)
        pos += len(it["emit"])
