"""QKV projection and attention of a layer in ONE launch (the default for models whose heads all have their own K / V
head, RMSNorm family) against the two separate launches (launch mode 2) and against the oracle.  The fused launch deals
the context to 3, 6 or 12 workgroups per head where the separate attention kernel uses ranges of 128 .. 1024 positions,
so the two agree to fp32 summation order (the projection's arithmetic is the same: the cache entries of a one-layer
model must be bitwise equal); both are held to the parity tests' bars against the oracle."""
import pytest
import torch

from paper_2405_04304_amd import binding as B
from oracle import disco_oracle as O
from workloads import synth as W

from test_gpu_parity import check_argmax, check_logits, dev, setup_pair

pytestmark = pytest.mark.gpu


def _verify(gm, gkv, ws, blk, mode):
    d = dev()
    M = len(blk)
    am = torch.zeros(16, dtype=torch.int32, device=d)
    lg = torch.empty(M, gm.shape.vocab, dtype=torch.float32, device=d)
    prev = B.disco_set_launch_mode(mode)
    try:
        B.disco_verify(gm, gkv, torch.tensor(blk, dtype=torch.int32, device=d), M, am, lg, ws)
        torch.cuda.synchronize()
    finally:
        B.disco_set_launch_mode(prev)
    return lg, am[:M].tolist()


# (shape, what the projection's launch looks like)
SHAPES = (
    (W.ModelShape("B", 2, 128, 2, 64, 2, 256, 512), "2 heads x 64: 6 workgroups per head of 32 rows"),
    (W.scaled_shape(W.CFG1_DRAFT, vocab=4096), "68M-class: 12 heads x 64, 6 workgroups per head"),
    (W.ModelShape("B", 2, 256, 2, 128, 2, 512, 512), "2 heads x 128: 12 workgroups per head of 32 rows"),
    (W.scaled_shape(W.CFG2_TARGET, n_layers=2, vocab=4096), "13B-class x 2 layers: 40 heads x 128, 6 workgroups per head of 64 rows"),
)


@pytest.mark.parametrize("si", range(len(SHAPES)))
def test_fused_launch_matches_separate_launches_and_oracle(si):
    shape, what = SHAPES[si]
    cases = ((0, 16, False), (40, 8, True), (200, 64, False), (1000, 16, True)) if si != 3 else ((0, 16, False), (1000, 64, True))
    for ctx, page_tokens, permute in cases:
        om, gm, okv, gkv, ws = setup_pair(shape, 4 + si, kv_ctx=ctx, capacity=ctx + 48, page_tokens=page_tokens, permute=permute,
                                          sigma=0.05 if si != 3 else 0.02)
        for M in (1, 5, 8, 11, 16):
            blk = W.make_tokens(50 + M, M, shape.vocab).tolist()
            lg0, am0 = _verify(gm, gkv, ws, blk, 0)
            B.disco_kv_rollback(gkv, ctx)
            lg2, am2 = _verify(gm, gkv, ws, blk, 2)
            ref = om.forward(blk, okv)
            tag = f"{what}, ctx {ctx}, pages of {page_tokens}, M {M}"
            check_logits(lg0, ref, "fused: " + tag)
            check_logits(lg2, ref, "separate: " + tag, quiet=True)
            check_argmax(am0, ref, "fused " + tag)
            scale = float(lg2.abs().max())
            assert float((lg0 - lg2).abs().max()) <= 2e-4 * scale, tag
            # an accepted prefix stays in the cache: the next block of this case runs on entries the fused launch wrote
            keep = ctx if M != 5 else ctx + 3
            B.disco_kv_rollback(gkv, keep)
            okv.rollback(keep)
            if keep != ctx:
                lg0, _ = _verify(gm, gkv, ws, blk[:2], 0)
                ref = om.forward(blk[:2], okv)
                check_logits(lg0, ref, "fused, after a kept prefix: " + tag)
                B.disco_kv_rollback(gkv, ctx)
                okv.rollback(ctx)


def test_fused_launch_writes_the_same_cache_entries():
    """One layer: the projection's inputs are the same in both structures, so q, K and V are bitwise the same."""
    d = dev()
    for shape in (W.scaled_shape(W.CFG1_DRAFT, n_layers=1, vocab=4096), W.scaled_shape(W.CFG2_TARGET, n_layers=1, vocab=4096)):
        for ctx, page_tokens in ((0, 16), (130, 8), (515, 64)):
            w = W.make_weights(shape, 9, "bf16")
            gm = B.DiscoModel(shape, w, d)
            fill = W.make_kv_fill(shape, ctx, 3).to(d) if ctx else None
            bufs = []
            for mode in (0, 2):
                gkv = B.DiscoKV(gm, ctx + 32, page_tokens)
                gkv.buf.zero_()
                gkv2 = gkv
                if fill is not None:
                    gkv.fill(fill)
                ws = gm.workspace(16, ctx + 32)
                _verify(gm, gkv2, ws, W.make_tokens(3, 13, shape.vocab).tolist(), mode)
                assert gkv.len == ctx + 13
                bufs.append(gkv.buf.clone())
            assert torch.equal(bufs[0], bufs[1]), (shape.d_model, ctx, page_tokens)


def _loop(gm, clf, fill, ctx, cap, tau, static_sl, ws, logits, tok0, force, mode):
    d = dev()
    kv = B.DiscoKV(gm, ctx + 32, 16)
    kv.fill(fill)
    steps = B.struct_tensor(B.ClfOut, 16, d)
    lo_d = B.struct_tensor(B.LoopOut, 1, d)
    lo_h = B.struct_tensor(B.LoopOut, 1, pinned=True)
    prev = B.disco_set_launch_mode(mode)
    try:
        B.disco_draft_loop(gm, kv, clf, tok0, tok0.numel(), cap, static_sl, 1.0, tau, force, logits, steps, lo_d, lo_h, ws)
        torch.cuda.synchronize()
    finally:
        B.disco_set_launch_mode(prev)
    lo = B.LoopOut.from_buffer_copy(lo_h.numpy().tobytes())
    return lo, [B.read_struct(B.ClfOut, steps, i) for i in range(cap)]


def test_fused_launch_in_the_draft_loop():
    """The draft loop's steps read the cache entries that the steps before them wrote through the fused launch, and a
    halted step's launches must leave the per-head counters untouched."""
    d = dev()
    shape = W.scaled_shape(W.CFG1_DRAFT, vocab=4096)
    gm = B.DiscoModel(shape, W.make_weights(shape, 3, "bf16"), d)
    clf = B.DiscoClf(W.make_classifier(100), d)
    ctx, cap = 300, 9
    fill = W.make_kv_fill(shape, ctx, 2).to(d)
    ws = gm.workspace(16, ctx + 32)
    logits = torch.empty(shape.vocab, dtype=torch.float32, device=d)
    force = torch.tensor([-1, 77, -1, -1, 5, -1, -1, -1, -1, -1], dtype=torch.int32, device=d)
    for tok0, tau, static_sl in ((torch.tensor([11, 12], dtype=torch.int32, device=d), 0.0, 0),
                                 (torch.tensor([11], dtype=torch.int32, device=d), 0.9, 0),
                                 (torch.tensor([11, 12], dtype=torch.int32, device=d), 2.0, 0),      # halts at once: 8 gated steps follow
                                 (torch.tensor([7], dtype=torch.int32, device=d), 0.5, 4)):
        (lo0, s0), (lo2, s2) = (_loop(gm, clf, fill, ctx, cap, tau, static_sl, ws, logits, tok0, force, mode) for mode in (0, 2))
        assert lo0.sl == lo2.sl >= 1 and list(lo0.block[:lo0.sl + 1]) == list(lo2.block[:lo2.sl + 1]), (tau, static_sl)
        for j in range(lo0.sl):
            assert s0[j].executed == s2[j].executed == 1 and s0[j].token == s2[j].token and s0[j].halt == s2[j].halt
            assert torch.allclose(torch.tensor(list(s0[j].feats)), torch.tensor(list(s2[j].feats)), rtol=1e-4, atol=1e-7)
            assert abs(s0[j].score - s2[j].score) < 1e-5


def test_a_wait_that_gives_up_is_reported_and_reinitialising_the_workspace_recovers():
    """The waits inside the fused launch are bounded.  With the limit forced to 'give up at once' from the host every
    kernel still runs to its end (all accesses stay inside the buffers whatever the data is), the workspace's abort word
    is set, and every result channel says so: NaN logits, -1 from the arg-max kernel, -1 lookahead from the loop.  The
    flag is sticky until disco_workspace_init; afterwards the same workspace gives the separate launches' results."""
    d = dev()
    shape = W.scaled_shape(W.CFG1_DRAFT, vocab=4096)
    gm = B.DiscoModel(shape, W.make_weights(shape, 3, "bf16"), d)
    clf = B.DiscoClf(W.make_classifier(100), d)
    ctx = 150
    fill = W.make_kv_fill(shape, ctx, 2).to(d)
    gkv = B.DiscoKV(gm, ctx + 32, 16)
    gkv.fill(fill)
    ws = gm.workspace(16, ctx + 32)
    blk = W.make_tokens(3, 6, shape.vocab).tolist()
    want, want_am = _verify(gm, gkv, ws, blk, 2)
    B.disco_kv_rollback(gkv, ctx)
    prev = B.disco_set_wait_limit(-1)
    try:
        lg, am = _verify(gm, gkv, ws, blk, 0)
        assert am == [-1] * len(blk) and bool(torch.isnan(lg).all())
        B.disco_kv_rollback(gkv, ctx)
    finally:
        assert B.disco_set_wait_limit(prev) == -1
    # sticky: the separate launches' results are flagged too, and so is a draft loop
    lg, am = _verify(gm, gkv, ws, blk, 2)
    assert am == [-1] * len(blk) and bool(torch.isnan(lg).all())
    B.disco_kv_rollback(gkv, ctx)
    logits = torch.empty(shape.vocab, dtype=torch.float32, device=d)
    lo, _ = _loop(gm, clf, fill, ctx, 4, 0.0, 0, ws, logits, torch.tensor([5], dtype=torch.int32, device=d), None, 0)
    assert lo.sl == -1
    # recovery
    B.lib().disco_workspace_init(gm.handle, ws.buf.data_ptr(), ws.nbytes, 16, ctx + 32, B._stream())
    lg, am = _verify(gm, gkv, ws, blk, 0)
    assert am == want_am
    assert float((lg - want).abs().max()) <= 2e-4 * float(want.abs().max())


def test_fused_launch_at_page_and_line_boundaries():
    """Which cache loads may go out before the per-head wait depends on where the block starts inside its page and inside
    a 128-byte line of the transposed V rows; sweep block starts around those boundaries, for page sizes below, at and
    above a line, against the separate launches (held to the oracle by the parity tests)."""
    d = dev()
    shape = W.ModelShape("B", 2, 128, 2, 64, 2, 256, 512)
    gm = B.DiscoModel(shape, W.make_weights(shape, 21, "bf16", sigma=0.08), d)
    cap = 560
    full = W.make_kv_fill(shape, 520, 5).to(d)
    for page_tokens in (4, 16, 64, 128):
        gkv = B.DiscoKV(gm, cap, page_tokens)
        ws = gm.workspace(16, cap)
        for ctx in (1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 255, 256, 257, 300, 383, 384, 511, 512, 520):
            fill = full[:, :, :ctx].contiguous()
            for M in (1, 16):
                blk = W.make_tokens(ctx + M, M, shape.vocab).tolist()
                out = []
                for mode in (0, 2):
                    gkv.fill(fill)
                    out.append(_verify(gm, gkv, ws, blk, mode))
                (lg0, am0), (lg2, am2) = out
                scale = float(lg2.abs().max())
                assert bool(torch.isfinite(lg0).all()) and float((lg0 - lg2).abs().max()) <= 2e-4 * scale, (page_tokens, ctx, M)


def test_fused_launch_over_other_head_layouts():
    """Head counts and widths that give 3, 6 and 12 workgroups per head, d_q different from d_model, odd head counts,
    pages of every size, permuted page order: the shared launch against the separate launches."""
    import random
    rng = random.Random(7)
    shapes = (W.ModelShape("B", 1, 256, 80, 64, 80, 256, 512),      # 15360 projection rows of 64-wide heads: 64-row workgroups, 3 per head
              W.ModelShape("B", 2, 128, 3, 64, 3, 128, 320),        # 6 per head, three heads, d_q 192 against d_model 128
              W.ModelShape("B", 2, 192, 5, 128, 5, 256, 320),       # 12 per head, five heads, d_q 640 against d_model 192
              W.ModelShape("B", 1, 64, 1, 128, 1, 64, 256))         # one head
    for si, shape in enumerate(shapes):
        gm = B.DiscoModel(shape, W.make_weights(shape, 30 + si, "bf16", sigma=0.08), dev())
        for _ in range(6):
            page_tokens = rng.choice((4, 8, 16, 32, 64, 128))
            ctx = rng.choice((0, 1, 17, 100, 129, 333, 640, 1500))
            M = rng.choice((1, 2, 3, 7, 8, 9, 16))
            cap = ctx + 32
            n_pages = (cap + page_tokens - 1) // page_tokens
            order = list(range(n_pages))
            rng.shuffle(order)
            gkv = B.DiscoKV(gm, cap, page_tokens, order)
            ws = gm.workspace(16, cap)
            fill = W.make_kv_fill(shape, ctx, 40 + si).to(dev()) if ctx else None
            blk = W.make_tokens(ctx + M, M, shape.vocab).tolist()
            out = []
            for mode in (0, 2):
                if fill is not None:
                    gkv.fill(fill)
                else:
                    B.disco_kv_rollback(gkv, 0)
                out.append(_verify(gm, gkv, ws, blk, mode))
            (lg0, am0), (lg2, am2) = out
            scale = float(lg2.abs().max())
            assert bool(torch.isfinite(lg0).all()) and float((lg0 - lg2).abs().max()) <= 2e-4 * scale, (si, page_tokens, ctx, M)
