"""Launch mode 1 (one cooperative launch per forward / per draft loop, grid barrier between the phases)
against the oracle and against launch mode 0 (one launch per phase).  Same tolerances as the parity tests:
logits within 2e-2 relative per row (and the 2e-3 regression bar), tokens equal off the flagged positions;
between the two modes the draft loop's tokens and lookahead must be identical and its features equal to
fp32 summation order (the K ranges of the split GEMMs differ between the modes)."""
import pytest
import torch

from paper_2405_04304_amd import binding as B
from oracle import disco_oracle as O
from workloads import synth as W

from test_gpu_parity import MARGIN, check_argmax, check_logits, dev, setup_pair

pytestmark = pytest.mark.gpu


@pytest.fixture
def mode1():
    prev = B.disco_set_launch_mode(1)
    yield
    B.disco_set_launch_mode(prev)


def test_launch_mode_argument():
    prev = B.disco_set_launch_mode(0)
    assert B.disco_set_launch_mode(prev) == 0
    assert B.disco_set_launch_mode(2) == prev            # 2: one launch per phase, nothing fused
    assert B.disco_set_launch_mode(prev) == 2
    for bad in (-1, 3):
        with pytest.raises(B.DiscoError):
            B.disco_set_launch_mode(bad)


def test_mode1_draft_step_and_verify_match_oracle(mode1):
    d = dev()
    shape = W.CFG1_DRAFT
    om, gm, okv, gkv, ws = setup_pair(shape, 0, kv_ctx=512, capacity=512 + 32)
    logits = torch.empty(shape.vocab, dtype=torch.float32, device=d)
    tok = int(W.make_tokens(3, 1, shape.vocab)[0])
    for step, n_in in enumerate((1, 2, 1)):
        toks = [tok] * n_in
        B.disco_draft_step(gm, gkv, torch.tensor(toks, dtype=torch.int32, device=d), n_in, logits, ws)
        torch.cuda.synchronize()
        ref = om.forward(toks, okv)[-1:]
        check_logits(logits[None], ref, f"mode 1: 68M draft step {step} n_in {n_in}")
        tok = O.argmax_lowest(ref[0])
    shape = W.scaled_shape(W.CFG2_TARGET, n_layers=2)
    om, gm, okv, gkv, ws = setup_pair(shape, 0, kv_ctx=1000, capacity=1000 + 24, permute=True)
    for M in (1, 8, 11, 16):
        blk = W.make_tokens(30 + M, M, shape.vocab).tolist()
        am = torch.zeros(16, dtype=torch.int32, device=d)
        lg = torch.empty(M, shape.vocab, dtype=torch.float32, device=d)
        B.disco_verify(gm, gkv, torch.tensor(blk, dtype=torch.int32, device=d), M, am, lg, ws)
        torch.cuda.synchronize()
        ref = om.forward(blk, okv)
        check_logits(lg, ref, f"mode 1: verify 13B-shape x2 layers M {M}")
        check_argmax(am[:M].tolist(), ref, "mode 1 verify")
        B.disco_kv_rollback(gkv, 1000)
        okv.rollback(1000)


def _loop(gm, clf, fill, ctx, cap, tau, static_sl, ws, logits, tok0, force=None):
    d = dev()
    kv = B.DiscoKV(gm, ctx + 32, 16)
    kv.fill(fill)
    steps = B.struct_tensor(B.ClfOut, 16, d)
    lo_d = B.struct_tensor(B.LoopOut, 1, d)
    lo_h = B.struct_tensor(B.LoopOut, 1, pinned=True)
    B.disco_draft_loop(gm, kv, clf, tok0, tok0.numel(), cap, static_sl, 1.0, tau, force, logits, steps, lo_d, lo_h, ws)
    torch.cuda.synchronize()
    lo = B.LoopOut.from_buffer_copy(lo_h.numpy().tobytes())
    assert kv.len == ctx + tok0.numel() + (static_sl or cap) - 1
    return lo, [B.read_struct(B.ClfOut, steps, i) for i in range(cap)]


def test_mode1_draft_loop_equals_mode0():
    d = dev()
    shape = W.scaled_shape(W.CFG1_DRAFT, vocab=4096)
    gm = B.DiscoModel(shape, W.make_weights(shape, 3, "bf16"), d)
    clf = B.DiscoClf(W.make_classifier(100), d)
    ctx, cap = 200, 7
    fill = W.make_kv_fill(shape, ctx, 2).to(d)
    ws = gm.workspace(16, ctx + 32)
    logits = torch.empty(shape.vocab, dtype=torch.float32, device=d)
    force = torch.tensor([-1, 77, -1, -1, 5, -1, -1, -1], dtype=torch.int32, device=d)
    for tok0, tau, static_sl in ((torch.tensor([11, 12], dtype=torch.int32, device=d), 0.0, 0),
                                 (torch.tensor([11], dtype=torch.int32, device=d), 0.9, 0),
                                 (torch.tensor([11, 12], dtype=torch.int32, device=d), 2.0, 0),
                                 (torch.tensor([7], dtype=torch.int32, device=d), 0.5, 4)):
        res = []
        for mode in (0, 1):
            prev = B.disco_set_launch_mode(mode)
            try:
                res.append(_loop(gm, clf, fill, ctx, cap, tau, static_sl, ws, logits, tok0, force))
            finally:
                B.disco_set_launch_mode(prev)
        (lo0, s0), (lo1, s1) = res
        assert lo0.sl == lo1.sl and list(lo0.block[:lo0.sl + 1]) == list(lo1.block[:lo1.sl + 1]), (tau, static_sl)
        for j in range(lo0.sl):
            assert s0[j].executed == s1[j].executed == 1 and s0[j].token == s1[j].token and s0[j].halt == s1[j].halt
            assert torch.allclose(torch.tensor(list(s0[j].feats)), torch.tensor(list(s1[j].feats)), rtol=1e-4, atol=1e-7)
            assert abs(s0[j].score - s1[j].score) < 1e-5
        for j in range(lo0.sl, cap):
            assert s1[j].executed == 0                      # the kernel left at the halting step


def test_mode1_iteration_driver_with_chunks_equals_mode0():
    """disco_iterate under launch mode 1: every chunk of draft steps is one cooperative launch that continues the block
    of the launch before (block_offset / open_end inside the kernel's own loop), the verification forward another.  The
    run must be the run of launch mode 0: same tokens, same blocks and acceptance counts, iteration by iteration."""
    from paper_2405_04304_amd.engine import SpecEngine
    d = dev()
    st = W.scaled_shape(W.CFG1_DRAFT, vocab=4096, n_layers=3)
    sd = W.scaled_shape(W.CFG1_DRAFT, vocab=4096)
    tw, dw = W.make_weights(st, 3, "bf16"), W.make_weights(sd, 13, "bf16")
    ot = O.Model(st, tw, kv_bf16=True)
    clf = W.make_classifier(100)
    prompt = W.make_prompt(2, 24, st.vocab).tolist()
    n_new = 40
    ref, _ = O.greedy_target(ot, prompt, n_new)
    force = {"mask": W.make_force_mask(5, n_new, 0.6), "tokens": ref}
    eng = SpecEngine(B.DiscoModel(st, tw, d), B.DiscoModel(sd, dw, d), B.DiscoClf(clf, d), max_ctx=96, page_tokens=16)
    runs = {}
    TAU = 0.52          # the seeded classifier's score grows with the position: short blocks first, then blocks up to the cap
    for mode in (0, 1):
        prev = B.disco_set_launch_mode(mode)
        try:
            for chunk in (2, 100):
                runs[(mode, chunk)] = eng.generate(prompt, n_new, {"mode": "disco", "tau": TAU, "sl_max": 7, "pos_mode": "absolute",
                                                                   "chunk": chunk}, force=force, trace=True)
        finally:
            B.disco_set_launch_mode(prev)
    base = runs[(0, 100)]
    print("[launch mode] lookahead histogram of the run:", base["sl_hist"], flush=True)
    assert any(it["sl"] >= 3 for it in base["iterations"])                           # blocks that span several chunks occur
    for key, r in runs.items():
        if key[0] == 0:
            assert r["tokens"] == base["tokens"]
            assert [(a["sl"], a["n"], a["block"]) for a in r["iterations"]] == [(b["sl"], b["n"], b["block"]) for b in base["iterations"]]
    # mode 1 against mode 0: equal unless the differing decision sits at a flagged margin (the two modes add in different
    # orders): a draft token whose two largest probabilities are within 2e-2 in logit units, or a score within 1e-3 of tau
    import math
    from loop_compare import first_difference
    assert runs[(1, 2)]["tokens"] == runs[(1, 100)]["tokens"]
    for chunk in (2, 100):
        a, b = runs[(1, chunk)], runs[(0, chunk)]
        for ai, bi in zip(a["iterations"], b["iterations"]):
            diff = first_difference(ai, bi)
            if diff is None:
                continue
            kind, j = diff
            assert kind in ("draft_token", "halt"), (chunk, diff)
            rec = bi["steps"][j - 1]
            if kind == "draft_token":
                assert math.log(rec.feats[0] / rec.feats[1]) < MARGIN, (chunk, diff)
            else:
                assert abs(rec.score - TAU) < 1e-3, (chunk, diff)
            break
