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
    with pytest.raises(B.DiscoError):
        B.disco_set_launch_mode(2)


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
