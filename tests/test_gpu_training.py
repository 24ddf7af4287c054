"""GPU parity of the classifier-training path (labelling run, training, F1) against the CPU oracle.

Training is an iteration in fp32 on the GPU and in float64 in the oracle: the same algorithm (standardised
features, mean binary cross-entropy, full-batch gradient steps), compared on its results: the loss
curve, the folded parameters, the scores they give, and the confusion counts except where a score lies
within 1e-3 of the threshold."""
import math

import pytest
import torch

from paper_2405_04304_amd import binding as B
from paper_2405_04304_amd.engine import SpecEngine
from oracle import disco_oracle as O
from workloads import synth as W

pytestmark = pytest.mark.gpu
MARGIN = 2e-2


def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


def _data(n, seed, hidden):
    g = torch.Generator().manual_seed(seed)
    feats = torch.rand(n, 12, generator=g)
    feats[:, 11] = torch.arange(1, n + 1, dtype=torch.float32)
    y = ((feats[:, 0] + 0.3 * feats[:, 10]) > 0.7).to(torch.int32)
    init = {"W1": torch.randn(hidden, 12, generator=g) * 0.1, "b1": torch.randn(hidden, generator=g) * 0.1,
            "w2": torch.randn(hidden, generator=g) * 0.1, "b2": torch.randn(1, generator=g) * 0.1}
    return feats, y, init


def _gpu_train(feats, y, init, epochs, lr):
    d = dev()
    clf = B.DiscoClf(init, d)
    loss = torch.zeros(max(epochs, 1), dtype=torch.float32, device=d)
    B.disco_clf_train(feats.to(d), y.to(d), feats.shape[0], clf.hidden, epochs, lr, clf.dev, loss)
    torch.cuda.synchronize()
    return clf, loss.cpu()[:epochs]


def _gpu_eval(clf, feats, y, tau):
    d = dev()
    scores = torch.zeros(feats.shape[0], dtype=torch.float32, device=d)
    counts = torch.zeros(4, dtype=torch.int32, device=d)
    B.disco_clf_eval(clf, feats.to(d), y.to(d), feats.shape[0], tau, scores, counts)
    torch.cuda.synchronize()
    return scores.cpu(), counts.cpu().tolist()


@pytest.mark.parametrize("n,hidden,epochs", [(400, 16, 200), (1000, 64, 150), (257, 100, 60), (2560, 64, 20)])
def test_train_matches_oracle(n, hidden, epochs):
    feats, y, init = _data(n, n + hidden, hidden)
    lr = 0.5
    want, losses = O.clf_train(feats, y, init, epochs, lr)
    clf, loss = _gpu_train(feats, y, init, epochs, lr)
    assert torch.allclose(loss.double(), torch.tensor(losses, dtype=torch.float64), rtol=2e-4, atol=2e-6)
    got = clf.params()
    for k in ("W1", "b1", "w2", "b2"):
        scale = float(want[k].abs().max())
        assert float((got[k] - want[k]).abs().max()) <= 2e-3 * scale + 1e-5, k
    scores, counts = _gpu_eval(clf, feats, y, 0.5)
    ev = O.clf_eval(feats, y, want, 0.5)
    ref_scores = torch.tensor(ev["scores"])
    assert float((scores.double() - ref_scores).abs().max()) < 1e-3
    near = int(((ref_scores - 0.5).abs() < 1e-3).sum())
    for got_c, want_c in zip(counts, (ev["tp"], ev["fp"], ev["fn"], ev["tn"])):
        assert abs(got_c - want_c) <= near
    assert sum(counts) == n
    assert loss[-1] < loss[0]
    # reproducible bit for bit
    clf2, loss2 = _gpu_train(feats, y, init, epochs, lr)
    assert torch.equal(clf2.dev, clf.dev) and torch.equal(loss2, loss)


def test_eval_counts_by_hand_and_zero_epochs():
    zero = {"W1": torch.zeros(4, 12), "b1": torch.zeros(4), "w2": torch.zeros(4), "b2": torch.zeros(1)}
    lab = torch.tensor([1, 1, 0, 1, 0], dtype=torch.int32)
    clf = B.DiscoClf(zero, dev())
    scores, counts = _gpu_eval(clf, torch.zeros(5, 12), lab, 0.5)
    assert scores.tolist() == [0.5] * 5 and counts == [3, 2, 0, 0]
    scores, counts = _gpu_eval(clf, torch.zeros(5, 12), lab, 0.51)
    assert counts == [0, 0, 3, 2]
    # zero epochs: the parameters come back folded but untrained
    feats, y, init = _data(50, 1, 8)
    clf0, _ = _gpu_train(feats, y, init, 0, 0.5)
    want, _ = O.clf_train(feats, y, init, 0, 0.5)
    got = clf0.params()
    for k in want:
        assert torch.allclose(got[k], want[k], rtol=1e-4, atol=1e-6), k
    with pytest.raises(B.DiscoError) as e:
        B.disco_clf_train(feats.to(dev()), y.to(dev()), 3000, 8, 1, 0.5, clf0.dev, None)
    assert e.value.code == B.ECAP


def test_label_run_training_and_trained_halting():
    """App. D.1 end to end on a small pair with 60 % forced agreement: labelling run -> training -> F1 ->
    the loop halting on the trained classifier, against the oracle running the same classifier."""
    st = W.ModelShape("B", 2, 128, 2, 64, 2, 256, 512)
    sd = W.ModelShape("B", 1, 128, 2, 64, 2, 256, 512)
    tw, dw = W.make_weights(st, 0, "bf16", sigma=0.1), W.make_weights(sd, 10, "bf16", sigma=0.1)
    ot, od = O.Model(st, tw, kv_bf16=True), O.Model(sd, dw, kv_bf16=True)
    init = W.make_classifier(100)
    prompt = W.make_prompt(1, 40, st.vocab).tolist()
    n_new = 160
    ref, margins = O.greedy_target(ot, prompt, n_new)
    force = {"mask": W.make_force_mask(5, n_new, 0.6), "tokens": ref}
    d = dev()
    gclf = B.DiscoClf(init, d)
    eng = SpecEngine(B.DiscoModel(st, tw, d), B.DiscoModel(sd, dw, d), gclf, max_ctx=n_new + 64, page_tokens=8)
    gg = eng.greedy(prompt, n_new)
    assert all(a == b or m < MARGIN for a, b, m in zip(gg, ref, margins))
    feats, labels, toks = eng.label_run(prompt, ref, force)
    run = O.label_run(od, prompt, ref, force)
    assert torch.allclose(feats.cpu(), run["feats"], rtol=2e-3, atol=1e-6)
    lab_gpu, lab_ref = labels.cpu().tolist(), run["labels"].tolist()
    assert all(a == b or m < MARGIN for a, b, m in zip(lab_gpu, lab_ref, run["margins"]))
    assert 0.4 < sum(lab_ref) / n_new < 0.8
    # train on the first 120 positions, validate on the rest
    n_tr = 120
    B.disco_clf_train(feats, labels, n_tr, gclf.hidden, 400, 0.5, gclf.dev, None)
    torch.cuda.synchronize()
    want, losses = O.clf_train(run["feats"][:n_tr], run["labels"][:n_tr], init, 400, 0.5)
    trained = gclf.params()
    sc_val, counts = _gpu_eval(gclf, feats[n_tr:].cpu(), labels[n_tr:].cpu(), 0.5)
    ev = O.clf_eval(run["feats"][n_tr:], run["labels"][n_tr:], want, 0.5)
    assert float((sc_val.double() - torch.tensor(ev["scores"])).abs().max()) < 5e-3
    f1 = 2 * counts[0] / max(2 * counts[0] + counts[1] + counts[2], 1)
    assert f1 > 0.95 and ev["f1"] > 0.95          # the forced logit makes acceptance predictable from the features
    # the loop with the GPU-trained classifier, against the oracle running the same parameters
    pol = {"mode": "disco", "tau": 0.5, "sl_max": 10, "pos_mode": "absolute"}
    orc = O.spec_decode(ot, od, trained, prompt, n_new, pol, force=force)
    gpu = eng.generate(prompt, n_new, pol, force=force, trace=True)
    assert orc["tokens"] == ref
    same = all((gi["sl"], gi["n"], gi["block"], gi["emit"]) == (oi["sl"], oi["n"], oi["block"], oi["emit"])
               for gi, oi in zip(gpu["iterations"], orc["iterations"]))
    flagged = any(m < MARGIN for it in orc["iterations"] for m in it["target_margins"]) or any(
        s["margin"] < MARGIN or abs(s["score"] - 0.5) <= 1e-3 for it in orc["iterations"] for s in it["steps"])
    assert same or flagged
    # trained halting adapts the lookahead: blocks end at the first doubtful token, so nearly every
    # drafted token but the last of a block is accepted, and fewer draft steps are spent than at the cap
    assert len(orc["sl_hist"]) > 2
    drafted = sum(it["sl"] for it in orc["iterations"]); accepted = sum(it["n"] for it in orc["iterations"])
    assert accepted >= 0.9 * (drafted - orc["n_iterations"])
    static10 = O.spec_decode(ot, od, trained, prompt, n_new, {"mode": "static", "gamma": 10}, force=force)
    assert orc["n_draft_forwards"] < 0.5 * static10["n_draft_forwards"]
    assert orc["n_iterations"] <= 1.15 * static10["n_iterations"]
