"""disco_iterate (one speculative iteration driven by the library) and the continued draft block it is built
on.  The chunk (draft steps enqueued between two looks at the halt flag) must not change anything: the runs
with chunk 1, 2, 3 and "whole loop at once" have to be identical, iteration by iteration, step record by step
record (bitwise: every chunking launches the same kernels on the same data), and one of them is compared
with the oracle's run by the parity tests' rule."""
import ctypes as C

import pytest
import torch

from paper_2405_04304_amd import binding as B
from paper_2405_04304_amd.engine import SpecEngine
from oracle import disco_oracle as O
from workloads import synth as W

from test_gpu_parity import _compare_runs, dev

pytestmark = pytest.mark.gpu


def _pair():
    st = W.ModelShape("B", 2, 128, 2, 64, 2, 256, 512)
    sd = W.ModelShape("B", 1, 128, 2, 64, 2, 256, 512)
    return st, sd, W.make_weights(st, 0, "bf16", sigma=0.1), W.make_weights(sd, 10, "bf16", sigma=0.1)


def _rec(s):
    return (s.executed, s.token, s.halt, tuple(s.feats), s.score)


def test_chunking_changes_nothing_and_run_matches_oracle():
    st, sd, tw, dw = _pair()
    ot, od = O.Model(st, tw, kv_bf16=True), O.Model(sd, dw, kv_bf16=True)
    clf = W.make_classifier(100)
    prompt = W.make_prompt(1, 40, st.vocab).tolist()
    n_new = 64
    ref, _ = O.greedy_target(ot, prompt, n_new)
    force = {"mask": W.make_force_mask(5, n_new, 0.6), "tokens": ref}
    d = dev()
    eng = SpecEngine(B.DiscoModel(st, tw, d), B.DiscoModel(sd, dw, d), B.DiscoClf(clf, d), max_ctx=160, page_tokens=8)
    policies = ({"mode": "disco", "tau": 0.8, "sl_max": 10, "pos_mode": "absolute"},
                {"mode": "static", "gamma": 5},
                {"mode": "oracle", "reference": ref, "sl_max": 9},
                {"mode": "ppl", "threshold": 8.0, "sl_max": 8},
                {"mode": "heuristic", "start": 4, "sl_max": 10})
    for pol in policies:
        runs = []
        for chunk in (100, 1, 2, 3, 0):
            runs.append(eng.generate(prompt, n_new, dict(pol, chunk=chunk), force=force, trace=True))
        base = runs[0]
        for r in runs[1:]:
            assert r["tokens"] == base["tokens"] and r["n_iterations"] == base["n_iterations"], pol["mode"]
            assert r["n_draft_forwards"] == base["n_draft_forwards"]
            for a, b in zip(r["iterations"], base["iterations"]):
                assert (a["sl"], a["n"], a["block"], a["emit"], a["ctx"]) == (b["sl"], b["n"], b["block"], b["emit"], b["ctx"])
                assert a["target_argmax"] == b["target_argmax"]
                if a["steps"] is not None:
                    assert [_rec(s) for s in a["steps"]] == [_rec(s) for s in b["steps"]]
        if pol["mode"] in ("disco", "static"):
            orc = O.spec_decode(ot, od, clf, prompt, n_new, pol, force=force)
            div = _compare_runs(runs[-1], orc, pol.get("tau"))
            if not div:
                assert runs[-1]["tokens"] == ref and runs[-1]["sl_hist"] == orc["sl_hist"]


def test_iterate_reports_enqueued_steps_and_cache_lengths():
    """A halt inside the first chunk must not enqueue the rest of the cap; both caches end where Fig. 1 says."""
    st, sd, tw, dw = _pair()
    d = dev()
    gt, gd = B.DiscoModel(st, tw, d), B.DiscoModel(sd, dw, d)
    clf = B.DiscoClf(W.make_classifier(100), d)
    ctx = 48
    kv_t, kv_d = B.DiscoKV(gt, 128, 8), B.DiscoKV(gd, 128, 8)
    kv_t.fill(W.make_kv_fill(st, ctx, 1).to(d))
    kv_d.fill(W.make_kv_fill(sd, ctx - 1, 2).to(d))          # the draft cache lacks two tokens
    ws_t, ws_d = gt.workspace(16, 128), gd.workspace(16, 128)
    bufs = B.iter_buffers(torch.zeros(16, dtype=torch.int32, device=d), torch.empty(sd.vocab, dtype=torch.float32, device=d),
                          B.struct_tensor(B.ClfOut, 16, d), B.struct_tensor(B.LoopOut, 1, d),
                          B.struct_tensor(B.LoopOut, 1, pinned=True), torch.zeros(16, dtype=torch.int32, device=d),
                          B.struct_tensor(B.AcceptOut, 1, d), B.struct_tensor(B.AcceptOut, 1, pinned=True))
    res = B.IterResult()
    # tau above every score: the first step halts (its token still counts), chunk 2 of cap 9 -> 2 steps enqueued
    B.disco_iterate(gt, kv_t, ws_t, gd, kv_d, ws_d, clf, [5, 9], 9, 0, 2, 1.0, 2.0, bufs, res)
    assert res.sl == 1 and res.draft_forwards == 1 and res.draft_steps_enqueued == 2
    assert res.block[0] == 9 and 0 <= res.n <= 1
    assert kv_t.len == ctx + res.n + 1 and kv_d.len == min(ctx - 1 + 2, ctx + res.n + 1)
    # tau below every score: no halt before the cap, chunks 2 + 2 + 1
    len_t = kv_t.len
    pend = [int(res.emit[res.n])] if kv_d.len == len_t else [int(res.emit[res.n - 1]), int(res.emit[res.n])]
    B.disco_iterate(gt, kv_t, ws_t, gd, kv_d, ws_d, clf, pend, 5, 0, 2, 1.0, -1.0, bufs, res)
    assert res.sl == 5 and res.draft_forwards == 5 and res.draft_steps_enqueued == 5
    assert kv_t.len == len_t + res.n + 1 and kv_d.len <= kv_t.len
    # no draft: the target decodes one token
    len_t = kv_t.len
    B.disco_iterate(gt, kv_t, ws_t, None, None, None, None, [int(res.emit[res.n])], 0, 0, 0, 1.0, 0.0, bufs, res)
    assert res.sl == 0 and res.n == 0 and res.draft_steps_enqueued == 0 and kv_t.len == len_t + 1
    with pytest.raises(B.DiscoError):
        B.disco_iterate(gt, kv_t, ws_t, gd, kv_d, ws_d, clf, [1, 2, 3], 4, 0, 0, 1.0, 0.0, bufs, res)


def test_continued_block_equals_one_call():
    """disco_draft_loop_ex with block_offset / open_end: 3 + 4 steps in two calls against 7 in one."""
    st, sd, tw, dw = _pair()
    d = dev()
    gd = B.DiscoModel(sd, dw, d)
    clf = B.DiscoClf(W.make_classifier(100), d)
    ctx, cap = 40, 7
    fill = W.make_kv_fill(sd, ctx, 2).to(d)
    ws = gd.workspace(16, 128)
    logits = torch.empty(sd.vocab, dtype=torch.float32, device=d)
    tok0 = torch.tensor([3, 4], dtype=torch.int32, device=d)
    out = []
    for split in (None, 3):
        kv = B.DiscoKV(gd, 128, 8)
        kv.fill(fill)
        steps = B.struct_tensor(B.ClfOut, 16, d)
        lo_d, lo_h = B.struct_tensor(B.LoopOut, 1, d), B.struct_tensor(B.LoopOut, 1, pinned=True)
        if split is None:
            B.disco_draft_loop_ex(gd, kv, clf, tok0, 2, cap, 0, 1.0, -1.0, logits, steps, lo_d, lo_h, ws)
        else:
            B.disco_draft_loop_ex(gd, kv, clf, tok0, 2, split, 0, 1.0, -1.0, logits, steps, lo_d, lo_h, ws, open_end=1)
            torch.cuda.synchronize()
            mid = B.LoopOut.from_buffer_copy(lo_h.numpy().tobytes())
            assert mid.sl == split and mid.halted == 0
            B.disco_draft_loop_ex(gd, kv, clf, lo_d.data_ptr() + 4 + 4 * split, 1, cap - split, 0, 1.0 + split, -1.0, logits,
                                  steps, lo_d, lo_h, ws, block_offset=split)
        torch.cuda.synchronize()
        lo = B.LoopOut.from_buffer_copy(lo_h.numpy().tobytes())
        assert lo.sl == cap and lo.halted == 1 and kv.len == ctx + 2 + cap - 1
        out.append((list(lo.block[:cap + 1]), [_rec(B.read_struct(B.ClfOut, steps, i)) for i in range(cap)]))
    assert out[0] == out[1]
    with pytest.raises(B.DiscoError):
        B.disco_draft_loop_ex(gd, kv, clf, tok0, 2, 10, 0, 1.0, -1.0, logits, steps, lo_d, lo_h, ws, block_offset=8)
