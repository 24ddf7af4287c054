"""GPU parity: the HIP path, called through the C boundary, against the CPU oracle on the same
seeded inputs.

Tolerances.  Logits: the workload statement allows max |x_gpu - x_ref| <= 2e-2 * max |x_ref| per row
(bf16 weights, fp32-vs-fp64 arithmetic); the kernels keep activations at fp32 grade (bf16 hi/lo
split), so the tests also hold a much tighter bound, 2e-3, to catch regressions.  Token ids and halt
bits must be identical except where the oracle flags a top-2 logit margin below 2e-2 or a classifier
score within 1e-3 of the threshold.  Integer results (acceptance, rollback lengths) are bit-exact."""
import ctypes as C
import math

import pytest
import torch

import paper_2405_04304_amd as D
from paper_2405_04304_amd import binding as B
from paper_2405_04304_amd.engine import SpecEngine
from oracle import disco_oracle as O
from workloads import synth as W

from loop_compare import compare_runs

pytestmark = pytest.mark.gpu

REL_TOL = 2e-2      # the stated bar
REL_TIGHT = 2e-3    # what the fp32-grade path actually holds
MARGIN = 2e-2


def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


def check_logits(got: torch.Tensor, ref: torch.Tensor, what="", tight=REL_TIGHT, quiet=False):
    got, ref = got.detach().cpu().double(), ref.double()
    assert got.shape == ref.shape
    assert torch.isfinite(got).all(), what
    worst = 0.0
    for r in range(ref.shape[0]):
        err = float((got[r] - ref[r]).abs().max())
        scale = float(ref[r].abs().max())
        worst = max(worst, err / scale)
        assert err <= REL_TOL * scale, (what, r, err, scale)
        assert err <= tight * scale, (what, "tight", r, err, scale)
    if not quiet:
        print(f"[parity] {what}: max rel err {worst:.3e} (bar {REL_TOL}, tight {tight})", flush=True)
    return worst


def check_argmax(got, ref_logits: torch.Tensor, what=""):
    for r, g in enumerate(got):
        want = O.argmax_lowest(ref_logits[r])
        if int(g) != want:
            assert O.top2_margin(ref_logits[r]) < MARGIN, (what, r, int(g), want)


def setup_pair(shape, seed, kv_ctx=0, kv_seed=2, page_tokens=16, permute=False, capacity=None,
               gain_jitter=0.0, sigma=0.02, weights=None):
    """Oracle model + GPU model on the same bf16 weights, optionally with the same pre-filled KV."""
    w = weights if weights is not None else W.make_weights(shape, seed, "bf16", sigma=sigma, gain_jitter=gain_jitter)
    om = O.Model(shape, w, kv_bf16=True)
    gm = B.DiscoModel(shape, w, dev())
    capacity = capacity or (kv_ctx + 64)
    okv = om.new_cache(capacity + 16)
    order = None
    if permute:
        n_pages = (capacity + page_tokens - 1) // page_tokens
        g = torch.Generator().manual_seed(77)
        order = torch.randperm(n_pages, generator=g).tolist()
    gkv = B.DiscoKV(gm, capacity, page_tokens, order)
    if kv_ctx:
        fill = W.make_kv_fill(shape, kv_ctx, kv_seed)
        okv.fill(fill)
        gkv.fill(fill.to(dev()))
    ws = gm.workspace(16, capacity)
    return om, gm, okv, gkv, ws


# ---- Eq. 2 kernel --------------------------------------------------------------------------------

def _run_classify(logits, clf_params, pos, tau, force=None, force_halt=0, multi=None):
    """multi=None runs both forms of the kernel (one workgroup / many workgroups with scratch) and
    checks that they agree before returning the first."""
    if multi is None:
        r1, x1 = _run_classify(logits, clf_params, pos, tau, force, force_halt, multi=False)
        r2, x2 = _run_classify(logits, clf_params, pos, tau, force, force_halt, multi=True)
        assert (r1.token, r1.halt, r1.executed) == (r2.token, r2.halt, r2.executed)
        assert torch.allclose(torch.tensor(list(r1.feats)), torch.tensor(list(r2.feats)), rtol=1e-5, atol=1e-7)
        assert (math.isnan(r1.score) and math.isnan(r2.score)) or abs(r1.score - r2.score) < 1e-6
        assert torch.equal(x1, x2)
        return r1, x1
    d = dev()
    x = logits.to(torch.float32).to(d).contiguous()
    clf = B.DiscoClf(clf_params, d) if clf_params is not None else None
    out = B.struct_tensor(B.ClfOut, 1, d)
    ft = torch.tensor([force if force is not None else -1], dtype=torch.int32, device=d)
    scratch = B.classify_scratch(d) if multi else None
    for _ in range(2 if multi else 1):       # a second call on the same scratch: the ticket word was left at zero
        xc = x.clone()
        B.disco_classify(clf, xc, xc.numel(), float(pos), float(tau), force_halt, out, force_token=ft, scratch=scratch)
        torch.cuda.synchronize()
    return B.read_struct(B.ClfOut, out), xc.cpu()


@pytest.mark.parametrize("V", [16, 1001, 4096, 32000, 49152])
def test_classify_matches_oracle(V):
    clf = W.make_classifier(100)
    g = torch.Generator().manual_seed(V)
    for trial in range(3):
        x = (torch.randn(V, generator=g) * (0.5 + trial)).to(torch.float32)
        pos = 1 + 7 * trial
        r, _ = _run_classify(x, clf, pos, 0.5)
        f = O.features(x.double(), pos)
        assert r.executed == 1
        assert r.token == f["token"]
        got = torch.tensor(list(r.feats), dtype=torch.float64)
        assert torch.allclose(got, f["feats"].double(), rtol=2e-5, atol=1e-6), (V, trial, got, f["feats"])
        c = O.classifier(f["feats"], clf)
        assert abs(r.score - c) < 1e-5
        if abs(c - 0.5) > 1e-3:
            assert r.halt == int(c < 0.5)


def test_classify_closed_forms_ties_and_forcing():
    clf = W.make_classifier(100)
    V = 32000
    # all-equal logits: p = 1/V, H = ln V, token 0; exercises the massive-tie path
    r, _ = _run_classify(torch.full((V,), 1.5), clf, 3, 0.5)
    assert r.token == 0
    assert all(abs(p - 1.0 / V) < 1e-9 for p in list(r.feats)[:10])
    assert abs(r.feats[10] - math.log(V)) < 1e-4
    # single spike
    x = torch.zeros(V)
    x[12345] = 5.0
    r, _ = _run_classify(x, clf, 3, 0.5)
    z = math.exp(5.0) + V - 1
    assert r.token == 12345 and abs(r.feats[0] - math.exp(5.0) / z) < 1e-6
    assert abs(r.feats[1] - 1 / z) < 1e-9 and abs(r.feats[9] - 1 / z) < 1e-9
    # forcing: the chosen logit becomes max + 4, in the features and in the logits buffer
    g = torch.Generator().manual_seed(3)
    x = torch.randn(V, generator=g)
    r, xb = _run_classify(x, clf, 9, 0.5, force=777)
    xo = x.double().clone()
    xo[777] = xo.max() + 4.0
    f = O.features(xo, 9)
    assert r.token == 777 and abs(float(xb[777]) - float(xo[777])) < 1e-6
    assert torch.allclose(torch.tensor(list(r.feats), dtype=torch.float64), f["feats"].double(), rtol=2e-5, atol=1e-6)
    # no classifier: score NaN, halt only when forced
    r, _ = _run_classify(x, None, 1, 0.5)
    assert math.isnan(r.score) and r.halt == 0
    r, _ = _run_classify(x, None, 1, 0.5, force_halt=1)
    assert r.halt == 1
    # tau above every score halts, tau = 0 never does
    assert _run_classify(x, clf, 1, 1.1)[0].halt == 1 and _run_classify(x, clf, 1, 0.0)[0].halt == 0


# ---- acceptance ------------------------------------------------------------------------------------

def test_accept_bit_exact():
    d = dev()
    g = torch.Generator().manual_seed(11)
    cases = [([100, 1, 2, 3, 4, 5], [1, 2, 3, 40, 50, 60])]          # Fig. 1: SL 5, three accepted
    cases += [([9], [4]), ([9, 1, 2], [7, 2, 3]), ([9, 1, 2], [1, 2, 3]), ([9, 1, 2, 3], [1, 5, 3, 4])]
    for _ in range(40):
        nb = int(torch.randint(1, 17, (1,), generator=g))
        a = torch.randint(0, 50, (nb,), generator=g).tolist()
        n_true = int(torch.randint(0, nb, (1,), generator=g))
        blk = [7] + a[:nb - 1]
        if n_true < nb - 1:
            blk[n_true + 1] = a[n_true] + 1                            # first mismatch after n_true
        cases.append((blk, a))
    out = B.struct_tensor(B.AcceptOut, 1, d)
    host = B.struct_tensor(B.AcceptOut, 1, pinned=True)
    for blk, a in cases:
        tb = torch.tensor(blk + [0] * (16 - len(blk)), dtype=torch.int32, device=d)
        ta = torch.tensor(a + [0] * (16 - len(a)), dtype=torch.int32, device=d)
        B.disco_accept(tb, ta, len(blk), out, host)
        torch.cuda.synchronize()
        r = B.read_struct(B.AcceptOut, out)
        rh = B.AcceptOut.from_buffer_copy(host.numpy().tobytes())
        n, emit = O.accept(blk, a)
        assert (r.n, list(r.emit[:r.n_emit])) == (n, emit) and r.n_emit == n + 1
        assert (rh.n, list(rh.emit[:rh.n_emit])) == (n, emit)


# ---- draft step -----------------------------------------------------------------------------------

SMALL_B = W.ModelShape("B", 2, 128, 2, 64, 2, 256, 512)
SMALL_B_GQA = W.ModelShape("B", 2, 256, 4, 64, 2, 288, 1008)
SMALL_A = W.ModelShape("A", 2, 128, 2, 64, 2, 256, 512, max_pos=512)
SMALL_A_MQA = W.ModelShape("A", 2, 256, 2, 128, 1, 512, 496, max_pos=512)


@pytest.mark.parametrize("shape,ctx,page,permute", [
    (SMALL_B, 0, 16, False), (SMALL_B, 37, 16, True), (SMALL_B_GQA, 300, 8, True),
    (SMALL_A, 129, 16, True), (SMALL_A_MQA, 200, 32, True)])
def test_draft_step_small_models(shape, ctx, page, permute):
    om, gm, okv, gkv, ws = setup_pair(shape, 5, kv_ctx=ctx, page_tokens=page, permute=permute, gain_jitter=0.2,
                                      sigma=0.05, capacity=ctx + 40)
    d = dev()
    logits = torch.empty(shape.vocab, dtype=torch.float32, device=d)
    toks = W.make_tokens(3, 12, shape.vocab).tolist()
    i = 0
    for n_in in (1, 2, 1, 1, 2, 1):                      # single-token steps and 2-token catch-up steps
        t = torch.tensor(toks[i:i + n_in], dtype=torch.int32, device=d)
        B.disco_draft_step(gm, gkv, t, n_in, logits, ws)
        torch.cuda.synchronize()
        ref = om.forward(toks[i:i + n_in], okv)[-1:]
        check_logits(logits[None], ref, f"draft_step {shape.family} ctx {okv.len} n_in {n_in}")
        i += n_in
        assert gkv.len == okv.len


@pytest.mark.parametrize("offset", [0.1, 0.5])
def test_layernorm_rows_with_a_mean(offset):
    """The LayerNorm of a forward is applied inside the consumer GEMM from per-tile sums: variance as E[h^2] - mean^2
    and the mean's share of the product removed afterwards, which lose digits as a row's mean grows against its
    spread.  Embedding rows with a common offset (mean / spread = 2 and 10 at sigma 0.05) must stay inside the
    regression bar; the stated bar holds far beyond."""
    shape = SMALL_A_MQA
    w = W.make_weights(shape, 7, "bf16", sigma=0.05, gain_jitter=0.2)
    w["tok_emb"] = (w["tok_emb"].float() + offset).to(torch.bfloat16)
    om, gm, okv, gkv, ws = setup_pair(shape, 7, kv_ctx=60, page_tokens=16, capacity=120, weights=w)
    d = dev()
    toks = W.make_tokens(9, 20, shape.vocab).tolist()
    am = torch.zeros(16, dtype=torch.int32, device=d)
    i = 0
    for M in (1, 5, 11):
        lg = torch.empty(M, shape.vocab, dtype=torch.float32, device=d)
        B.disco_verify(gm, gkv, torch.tensor(toks[i:i + M], dtype=torch.int32, device=d), M, am, lg, ws)
        torch.cuda.synchronize()
        ref = om.forward(toks[i:i + M], okv)
        check_logits(lg, ref, f"LayerNorm rows with mean offset {offset}, M {M}")
        i += M


@pytest.mark.parametrize("ctx", [512, 1024, 2048])
def test_draft_step_68m_shape(ctx):
    shape = W.CFG1_DRAFT
    om, gm, okv, gkv, ws = setup_pair(shape, 0, kv_ctx=ctx, capacity=ctx + 32)
    d = dev()
    logits = torch.empty(shape.vocab, dtype=torch.float32, device=d)
    clf = W.make_classifier(100)
    gclf = B.DiscoClf(clf, d)
    out = B.struct_tensor(B.ClfOut, 1, d)
    tok = int(W.make_tokens(3, 1, shape.vocab)[0])
    for step in range(3):
        t = torch.tensor([tok], dtype=torch.int32, device=d)
        B.disco_draft_step(gm, gkv, t, 1, logits, ws)
        B.disco_classify(gclf, logits, shape.vocab, float(step + 1), 0.5, 0, out)
        torch.cuda.synchronize()
        ref = om.forward([tok], okv)
        check_logits(logits[None], ref, f"68M draft step ctx {ctx}+{step}")
        r = B.read_struct(B.ClfOut, out)
        f = O.features(ref[0], step + 1)
        if f["margin"] >= MARGIN:
            assert r.token == f["token"]
        assert torch.allclose(torch.tensor(list(r.feats)), f["feats"], rtol=1e-3, atol=1e-6)
        c = O.classifier(f["feats"], clf)
        assert abs(r.score - c) < 1e-4
        if abs(c - 0.5) > 1e-3:
            assert r.halt == int(c < 0.5)
        tok = f["token"]


# ---- verification block -----------------------------------------------------------------------------

def _verify_case(shape, seed, ctx, ms, page=16, permute=True, what="", weights=None, jitter=0.0):
    om, gm, okv, gkv, ws = setup_pair(shape, seed, kv_ctx=ctx, page_tokens=page, permute=permute,
                                      capacity=ctx + 24, gain_jitter=jitter, weights=weights)
    d = dev()
    for M in ms:
        blk = W.make_tokens(30 + M, M, shape.vocab).tolist()
        tb = torch.tensor(blk, dtype=torch.int32, device=d)
        am = torch.zeros(16, dtype=torch.int32, device=d)
        lg = torch.empty(M, shape.vocab, dtype=torch.float32, device=d)
        B.disco_verify(gm, gkv, tb, M, am, lg, ws)
        torch.cuda.synchronize()
        assert gkv.len == ctx + M
        ref = om.forward(blk, okv)
        check_logits(lg, ref, f"verify {what} ctx {ctx} M {M}")
        check_argmax(am[:M].tolist(), ref, what)
        # arg-max without the optional logits output must be the same tokens
        B.disco_kv_rollback(gkv, ctx)
        am2 = torch.zeros(16, dtype=torch.int32, device=d)
        B.disco_verify(gm, gkv, tb, M, am2, None, ws)
        torch.cuda.synchronize()
        assert am2[:M].tolist() == am[:M].tolist()
        B.disco_kv_rollback(gkv, ctx)
        okv.rollback(ctx)
    return om, gm, okv, gkv, ws


def test_verify_small_models_all_block_lengths():
    _verify_case(SMALL_B, 6, 100, range(1, 17), page=8, what="B small", jitter=0.2)
    _verify_case(SMALL_A_MQA, 7, 130, (1, 3, 8, 9, 16), page=16, what="A MQA small", jitter=0.2)
    _verify_case(SMALL_B_GQA, 8, 0, (1, 5, 16), page=16, what="B GQA empty cache")


def test_verify_13b_shape_two_layers():
    shape = W.scaled_shape(W.CFG2_TARGET, n_layers=2)
    _verify_case(shape, 0, 1024, (1, 2, 4, 8, 11), what="13B-shape x2 layers")
    _verify_case(shape, 0, 1000, (11,), page=16, what="13B-shape ragged ctx")


def test_verify_mqa_code_model_shape_two_layers():
    shape = W.scaled_shape(W.CFG3_TARGET, n_layers=2, max_pos=2304)
    _verify_case(shape, 0, 2048, (1, 11), what="15B-MQA-shape x2 layers")


def test_verify_rollback_causality_and_m1_equals_draft_step():
    shape = SMALL_B_GQA
    om, gm, okv, gkv, ws = setup_pair(shape, 9, kv_ctx=50, page_tokens=8, permute=True, capacity=120)
    d = dev()
    a = torch.tensor([5, 6, 7, 8, 9, 10, 11, 12, 13], dtype=torch.int32, device=d)
    b = torch.tensor([5, 6, 70, 80, 90, 1, 2, 3, 4], dtype=torch.int32, device=d)
    am = torch.zeros(16, dtype=torch.int32, device=d)
    la = torch.empty(9, shape.vocab, dtype=torch.float32, device=d)
    lb = torch.empty_like(la)
    lf = torch.empty_like(la)
    B.disco_verify(gm, gkv, a, 9, am, la, ws)
    B.disco_kv_rollback(gkv, 50)
    B.disco_kv_rollback(gkv, 50)                          # idempotent
    assert gkv.len == 50 and gkv.pages_in_use == 7
    B.disco_verify(gm, gkv, b, 9, am, lb, ws)
    torch.cuda.synchronize()
    assert torch.equal(la[:2], lb[:2])                    # rows that see equal prefixes: bitwise equal
    assert not torch.equal(la[2], lb[2])
    # fresh cache, block B only: the stale suffix left by block A must be dead
    om2, gm2, okv2, gkv2, ws2 = setup_pair(shape, 9, kv_ctx=50, page_tokens=8, permute=True, capacity=120)
    B.disco_verify(gm2, gkv2, b, 9, am, lf, ws2)
    torch.cuda.synchronize()
    assert torch.equal(lf, lb)
    with pytest.raises(B.DiscoError) as e:
        B.disco_kv_rollback(gkv, 60)
    assert e.value.code == B.ESTATE
    # a one-token verification block is the same computation as a draft step
    B.disco_kv_rollback(gkv, 50)
    l1 = torch.empty(1, shape.vocab, dtype=torch.float32, device=d)
    B.disco_verify(gm, gkv, b, 1, am, l1, ws)
    B.disco_kv_rollback(gkv, 50)
    l2 = torch.empty(shape.vocab, dtype=torch.float32, device=d)
    B.disco_draft_step(gm, gkv, b, 1, l2, ws)
    torch.cuda.synchronize()
    assert torch.equal(l1[0], l2)
    # capacity errors come from the host and leave the length alone
    B.disco_kv_rollback(gkv, 50)
    with pytest.raises(B.DiscoError) as e:
        big = B.DiscoKV(gm, 16, 16)
        B.disco_verify(gm, big, a, 9, am, None, ws)
        B.disco_verify(gm, big, a, 9, am, None, ws)
    assert e.value.code == B.ECAP


# ---- the loop ----------------------------------------------------------------------------------------

def _compare_runs(gpu, orc, tau=None):
    """Token streams and schedules must agree up to the first position where the oracle flags the very
    decision that differs (loop_compare); returns whether the runs diverged there."""
    def feats_agree(gi, oi):
        if gi.get("steps") is not None:
            for gs, os_ in zip(gi["steps"], oi["steps"]):
                assert torch.allclose(torch.tensor(list(gs.feats)), os_["feats"], rtol=2e-3, atol=1e-5)
                assert abs(gs.score - os_["score"]) < 1e-3

    near = (lambda s: abs(s["score"] - tau) <= 1e-3) if tau is not None else None
    return compare_runs(gpu, orc, near, feats_agree) is not None


def test_loop_cfg0_matches_oracle_and_greedy():
    shape_t, shape_d = W.CFG0_TARGET, W.CFG0_DRAFT
    tw = W.make_weights(shape_t, 0, "bf16")
    dw = W.early_exit_draft(tw, 1)
    ot, od = O.Model(shape_t, tw, kv_bf16=True), O.Model(shape_d, dw, kv_bf16=True)
    clf = W.make_classifier(100)
    prompt = W.make_prompt(1, 32, shape_t.vocab).tolist()
    ref, margins = O.greedy_target(ot, prompt, 64)
    d = dev()
    gt, gd = B.DiscoModel(shape_t, tw, d), B.DiscoModel(shape_d, dw, d)
    eng = SpecEngine(gt, gd, B.DiscoClf(clf, d), max_ctx=112, page_tokens=16)
    # GPU greedy == oracle greedy up to the first flagged position
    gg = eng.greedy(prompt, 64)
    for p, (a, b) in enumerate(zip(gg, ref)):
        if a != b:
            assert margins[p] < MARGIN, (p, a, b, margins[p])
            break
    n_div = 0
    for pol in ([{"mode": "static", "gamma": g} for g in (0, 1, 5, 8)]
                + [{"mode": "disco", "tau": t, "sl_max": 8, "pos_mode": pm}
                   for t in (0.5, 0.55, 0.6, 0.9) for pm in ("absolute", "block")]):
        orc = O.spec_decode(ot, od, clf, prompt, 64, pol)
        gpu = eng.generate(prompt, 64, pol, trace=True)
        assert len(gpu["tokens"]) == 64
        n_div += _compare_runs(gpu, orc, pol.get("tau"))
        # whatever the schedule, the GPU's speculative text equals the GPU's own greedy text
        # unless a flagged position intervened
        if gpu["tokens"] != gg:
            p = next(i for i, (a, b) in enumerate(zip(gpu["tokens"], gg)) if a != b)
            assert margins[p] < MARGIN
    print(f"[parity] cfg0 loop: {n_div} of 12 policy runs diverged at a flagged position", flush=True)


def test_cfg0_fp32_statement_against_bf16_storage():
    """The tiny pair is stated with fp32 weights; the library stores matrices and KV entries as bf16 (the
    reading: bf16 storage is part of the design and applies to the tiny pair too).  The oracle on the fp32 weights with an fp32 cache, against the
    GPU on the bf16-rounded weights with a bf16 cache, teacher-forced along the oracle's own greedy text:
    every row of logits within the stated 2e-2 relative, every arg-max equal except where the oracle flags a
    top-2 margin below 2e-2."""
    shape = W.CFG0_TARGET
    w32 = W.make_weights(shape, 0, "f32")
    o32 = O.Model(shape, w32, kv_bf16=False)
    prompt = W.make_prompt(1, 32, shape.vocab).tolist()
    ref_tokens, _ = O.greedy_target(o32, prompt, 64)
    seq = prompt + ref_tokens
    okv = o32.new_cache(len(seq) + 1)
    ref = torch.cat([o32.forward(seq[i:i + 16], okv) for i in range(0, len(seq), 16)])
    d = dev()
    gm = B.DiscoModel(shape, {k: (v.to(torch.bfloat16) if v.dim() == 2 else v) for k, v in w32.items()}, d)
    gkv = B.DiscoKV(gm, len(seq) + 16, 16)
    ws = gm.workspace(16, len(seq) + 16)
    am = torch.zeros(16, dtype=torch.int32, device=d)
    tt = torch.tensor(seq, dtype=torch.int32, device=d)
    rows, toks = [], []
    for i in range(0, len(seq), 16):
        lg = torch.empty(16, shape.vocab, dtype=torch.float32, device=d)
        B.disco_verify(gm, gkv, tt.data_ptr() + 4 * i, 16, am, lg, ws)
        torch.cuda.synchronize()
        rows.append(lg.cpu())
        toks += am.tolist()
    got = torch.cat(rows)
    worst, n_flag = 0.0, 0
    for r in range(len(seq)):
        err = float((got[r].double() - ref[r].double()).abs().max())
        scale = float(ref[r].abs().max())
        worst = max(worst, err / scale)
        assert err <= REL_TOL * scale, (r, err, scale)
        if toks[r] != O.argmax_lowest(ref[r]):
            assert O.top2_margin(ref[r]) < MARGIN, (r, toks[r])
            n_flag += 1
    print(f"[parity] cfg0 fp32 statement vs bf16 storage: max rel err {worst:.3e} (bar {REL_TOL}), "
          f"{n_flag} arg-max differences, all at flagged rows", flush=True)


def test_loop_forced_acceptance_small_pair():
    """Independent draft, 60 % forced agreement (the full-loop workload's recipe), small shapes."""
    st = W.ModelShape("B", 2, 128, 2, 64, 2, 256, 512)
    sd = W.ModelShape("B", 1, 128, 2, 64, 2, 256, 512)
    tw, dw = W.make_weights(st, 0, "bf16", sigma=0.1), W.make_weights(sd, 10, "bf16", sigma=0.1)
    ot, od = O.Model(st, tw, kv_bf16=True), O.Model(sd, dw, kv_bf16=True)
    clf = W.make_classifier(100)
    prompt = W.make_prompt(1, 40, st.vocab).tolist()
    n_new = 96
    ref, margins = O.greedy_target(ot, prompt, n_new)
    force = {"mask": W.make_force_mask(5, n_new, 0.6), "tokens": ref}
    d = dev()
    eng = SpecEngine(B.DiscoModel(st, tw, d), B.DiscoModel(sd, dw, d), B.DiscoClf(clf, d), max_ctx=160, page_tokens=8)
    for pol in ({"mode": "static", "gamma": 5}, {"mode": "disco", "tau": 0.7, "sl_max": 10, "pos_mode": "block"},
                {"mode": "disco", "tau": 0.9, "sl_max": 10, "pos_mode": "absolute"}):
        orc = O.spec_decode(ot, od, clf, prompt, n_new, pol, force=force)
        assert orc["tokens"] == ref
        gpu = eng.generate(prompt, n_new, pol, force=force, trace=True)
        div = _compare_runs(gpu, orc, pol.get("tau"))
        if not div:
            assert gpu["tokens"] == ref and gpu["sl_hist"] == orc["sl_hist"]
            assert gpu["n_draft_forwards"] == sum(it["sl"] for it in orc["iterations"])
        assert sum(it["n"] for it in gpu["iterations"]) > n_new // 4      # forcing does produce acceptance


def _teacher_forced(st, sd, tw, dw, clf_p, prompt, n_new, pol, force=None):
    """Every call of every iteration of the oracle's run is repeated on the GPU with the ORACLE's inputs
    (its pending tokens, its draft tokens, its block), and every output is compared: draft logits, Eq. 2
    features, score, token and halt bit of every draft step; the target's arg-max of every block row; the
    acceptance result.  A flagged decision is skipped, and since the next call is fed the oracle's tokens
    again the comparison goes on to the end of the run instead of stopping there."""
    d = dev()
    ot, od = O.Model(st, tw, kv_bf16=True), O.Model(sd, dw, kv_bf16=True)
    orc = O.spec_decode(ot, od, clf_p, prompt, n_new, pol, force=force)
    gt, gd = B.DiscoModel(st, tw, d), B.DiscoModel(sd, dw, d)
    clf = B.DiscoClf(clf_p, d)
    cap_ctx = len(prompt) + n_new + 32
    kv_t, kv_d = B.DiscoKV(gt, cap_ctx, 16), B.DiscoKV(gd, cap_ctx, 16)
    ws_t, ws_d = gt.workspace(16, cap_ctx), gd.workspace(16, cap_ctx)
    am = torch.zeros(16, dtype=torch.int32, device=d)
    pre = torch.tensor(prompt[:-1], dtype=torch.int32, device=d)
    for model, kv, ws in ((gt, kv_t, ws_t), (gd, kv_d, ws_d)):
        for i in range(0, len(prompt) - 1, 16):
            B.disco_verify(model, kv, pre.data_ptr() + 4 * i, min(16, len(prompt) - 1 - i), am, None, ws)
    # the oracle's draft model replays its own run so that its logits are at hand for every step
    okv_d = od.new_cache(cap_ctx)
    od.prefill(list(prompt[:-1]), okv_d, 64)
    logits = torch.empty(sd.vocab, dtype=torch.float32, device=d)
    out = B.struct_tensor(B.ClfOut, 1, d)
    acc = B.struct_tensor(B.AcceptOut, 1, d)
    seq = list(prompt)
    tau = pol.get("tau")
    n_steps = n_skipped = 0
    for it in orc["iterations"]:
        emitted = len(seq) - len(prompt)
        sl, block = it["sl"], it["block"]
        assert kv_d.len == okv_d.len
        feed = seq[kv_d.len:]                                # pending tokens of the first draft call (1 or 2)
        for j, stp in enumerate(it["steps"], start=1):
            tin = torch.tensor(feed, dtype=torch.int32, device=d)
            B.disco_draft_step(gd, kv_d, tin, len(feed), logits, ws_d)
            ref = od.forward(feed, okv_d)[-1:]
            ft = None
            if force is not None and bool(force["mask"][emitted + j - 1]):
                ft = torch.tensor([int(force["tokens"][emitted + j - 1])], dtype=torch.int32, device=d)
            pos = float(emitted + j) if pol.get("pos_mode", "absolute") == "absolute" else float(j)
            B.disco_classify(clf, logits, sd.vocab, pos, tau if tau is not None else 0.0, 0, out, force_token=ft)
            torch.cuda.synchronize()
            if ft is None:
                check_logits(logits[None], ref, f"teacher-forced draft step, iteration ctx {it['ctx']} step {j}", quiet=True)
            r = B.read_struct(B.ClfOut, out)
            n_steps += 1
            if stp["margin"] >= MARGIN:
                assert r.token == stp["token"], (it["ctx"], j, r.token, stp["token"])
            else:
                n_skipped += 1
            assert torch.allclose(torch.tensor(list(r.feats)), stp["feats"], rtol=2e-3, atol=1e-5)
            if tau is not None and stp["score"] is not None:
                assert abs(r.score - stp["score"]) < 1e-3
                if abs(stp["score"] - tau) > 1e-3:
                    assert bool(r.halt & 1) == (stp["score"] < tau)
            feed = [stp["token"]]                            # the ORACLE's token goes in next
        tb = torch.tensor(block, dtype=torch.int32, device=d)
        assert kv_t.len == it["ctx"]
        B.disco_verify(gt, kv_t, tb, sl + 1, am, None, ws_t)
        # acceptance on the oracle's block and the oracle's arg-max: bit-exact; on the GPU's arg-max: equal
        # rows except flagged ones
        got = am[:sl + 1].tolist()
        for r_, (g_, o_) in enumerate(zip(got, it["target_argmax"])):
            if g_ != o_:
                assert it["target_margins"][r_] < MARGIN, (it["ctx"], r_, g_, o_)
        ta = torch.tensor(it["target_argmax"], dtype=torch.int32, device=d)
        B.disco_accept(tb, ta, sl + 1, acc)
        a = B.read_struct(B.AcceptOut, acc)
        assert a.n == it["n"] and list(a.emit[:a.n + 1])[:len(it["emit"])] == it["emit"]
        seq += it["emit"]
        len_t = it["ctx"] + it["n"] + 1
        B.disco_kv_rollback(kv_t, len_t)
        if kv_d.len > len_t:                                 # the draft keeps what the target kept
            B.disco_kv_rollback(kv_d, len_t)
            okv_d.rollback(len_t)
    assert seq[len(prompt):] == orc["tokens"]
    return len(orc["iterations"]), n_steps, n_skipped


def test_loop_teacher_forced_every_iteration_compared():
    # the tiny LayerNorm / GELU pair with the early-exit draft, DISCO halting in both position modes
    st, sd = W.CFG0_TARGET, W.CFG0_DRAFT
    tw = W.make_weights(st, 0, "bf16")
    dw = W.early_exit_draft(tw, 1)
    clf = W.make_classifier(100)
    prompt = W.make_prompt(1, 32, st.vocab).tolist()
    for pol in ({"mode": "disco", "tau": 0.6, "sl_max": 8, "pos_mode": "block"},
                {"mode": "disco", "tau": 0.55, "sl_max": 8, "pos_mode": "absolute"}, {"mode": "static", "gamma": 5}):
        n_it, n_st, n_sk = _teacher_forced(st, sd, tw, dw, clf, prompt, 64, pol)
        print(f"[parity] teacher-forced cfg0 {pol}: {n_it} iterations, {n_st} draft steps compared, {n_sk} tokens at flagged margins", flush=True)
    # RMSNorm / rotary / SwiGLU pair with an independent draft and 60 % forced agreement
    st = W.ModelShape("B", 2, 128, 2, 64, 2, 256, 512)
    sd = W.ModelShape("B", 1, 128, 2, 64, 2, 256, 512)
    tw, dw = W.make_weights(st, 0, "bf16", sigma=0.1), W.make_weights(sd, 10, "bf16", sigma=0.1)
    prompt = W.make_prompt(1, 40, st.vocab).tolist()
    ref, _ = O.greedy_target(O.Model(st, tw, kv_bf16=True), prompt, 96)
    force = {"mask": W.make_force_mask(5, 96, 0.6), "tokens": ref}
    n_it, n_st, n_sk = _teacher_forced(st, sd, tw, dw, clf, prompt, 96, {"mode": "disco", "tau": 0.7, "sl_max": 10, "pos_mode": "block"},
                                       force=force)
    print(f"[parity] teacher-forced forced-acceptance pair: {n_it} iterations, {n_st} draft steps compared, {n_sk} at flagged margins", flush=True)


def test_loop_reference_lookahead_matches_oracle():
    """Sec. 3, 'Finding the optimal SL per iteration': draft until the first token that leaves the target's
    greedy text; that token stays out of the block, so every drafted token is accepted."""
    st = W.ModelShape("B", 2, 128, 2, 64, 2, 256, 512)
    sd = W.ModelShape("B", 1, 128, 2, 64, 2, 256, 512)
    tw, dw = W.make_weights(st, 0, "bf16", sigma=0.1), W.make_weights(sd, 10, "bf16", sigma=0.1)
    ot, od = O.Model(st, tw, kv_bf16=True), O.Model(sd, dw, kv_bf16=True)
    clf = W.make_classifier(100)
    prompt = W.make_prompt(1, 40, st.vocab).tolist()
    n_new = 96
    ref, margins = O.greedy_target(ot, prompt, n_new)
    force = {"mask": W.make_force_mask(5, n_new, 0.6), "tokens": ref}
    d = dev()
    eng = SpecEngine(B.DiscoModel(st, tw, d), B.DiscoModel(sd, dw, d), B.DiscoClf(clf, d), max_ctx=160, page_tokens=8)
    for cap in (15, 3):
        pol = {"mode": "oracle", "reference": ref, "sl_max": cap}
        orc = O.spec_decode(ot, od, clf, prompt, n_new, pol, force=force)
        assert orc["tokens"] == ref and all(it["n"] == it["sl"] for it in orc["iterations"])
        gpu = eng.generate(prompt, n_new, pol, force=force, trace=True)
        div = _compare_runs(gpu, orc)
        if not div:
            assert gpu["tokens"] == ref and gpu["sl_hist"] == orc["sl_hist"]
            assert gpu["n_draft_forwards"] == orc["n_draft_forwards"]
            assert all(it["n"] == it["sl"] <= cap for it in gpu["iterations"])
            # the step whose token left the reference is recorded with bit 1 of halt set
            for gi, oi in zip(gpu["iterations"], orc["iterations"]):
                assert len(gi["steps"]) == len(oi["steps"])
                for gs, os_ in zip(gi["steps"], oi["steps"]):
                    assert gs.token == os_["token"] and bool(gs.halt & 2) == bool(os_.get("mismatch", False))
        assert max(gpu["sl_hist"]) > 1 and min(gpu["sl_hist"]) == 0          # lookaheads do vary
    # static lookahead can never accept more than the reference lookahead allows (its definition)
    st5 = eng.generate(prompt, n_new, {"mode": "static", "gamma": 5}, force=force)
    orc15 = O.spec_decode(ot, od, clf, prompt, n_new, {"mode": "oracle", "reference": ref, "sl_max": 15}, force=force)
    assert st5["n_iterations"] >= orc15["n_iterations"]


def test_loop_rule_based_baselines_match_oracle():
    """The two rule-based lookahead baselines (Sec. 2 footnote: a lookahead that follows the previous
    iteration's acceptance; App. F: a perplexity threshold).  Schedules, blocks and texts must equal the
    oracle's up to a flagged position; under the perplexity rule a step whose value is within 1e-3
    (relative) of the threshold is flagged too, and the per-step perplexities must agree."""
    st = W.ModelShape("B", 2, 128, 2, 64, 2, 256, 512)
    sd = W.ModelShape("B", 1, 128, 2, 64, 2, 256, 512)
    tw, dw = W.make_weights(st, 0, "bf16", sigma=0.1), W.make_weights(sd, 10, "bf16", sigma=0.1)
    ot, od = O.Model(st, tw, kv_bf16=True), O.Model(sd, dw, kv_bf16=True)
    clf = W.make_classifier(100)
    prompt = W.make_prompt(1, 40, st.vocab).tolist()
    n_new = 96
    ref, margins = O.greedy_target(ot, prompt, n_new)
    force = {"mask": W.make_force_mask(5, n_new, 0.6), "tokens": ref}
    d = dev()
    eng = SpecEngine(B.DiscoModel(st, tw, d), B.DiscoModel(sd, dw, d), B.DiscoClf(clf, d), max_ctx=160, page_tokens=8)
    heur = {"mode": "heuristic", "start": 5, "up": 2, "down": 1, "sl_max": 10}
    orc = O.spec_decode(ot, od, clf, prompt, n_new, heur, force=force)
    gpu = eng.generate(prompt, n_new, heur, force=force, trace=True)
    if not _compare_runs(gpu, orc):
        assert gpu["tokens"] == ref and gpu["sl_hist"] == orc["sl_hist"] and len(gpu["sl_hist"]) > 3
    # thresholds from the oracle's own range of values: the median, and a high and a low quantile
    probe = O.spec_decode(ot, od, clf, prompt, n_new, {"mode": "ppl", "threshold": 1e30, "sl_max": 10}, force=force)
    vals = sorted(s["ppl"] for it in probe["iterations"] for s in it["steps"])
    for q in (0.5, 0.85, 0.15):
        thr = vals[int(q * (len(vals) - 1))] * 1.01
        pol = {"mode": "ppl", "threshold": thr, "sl_max": 10}
        orc = O.spec_decode(ot, od, clf, prompt, n_new, pol, force=force)
        gpu = eng.generate(prompt, n_new, pol, force=force, trace=True)
        def ppl_agree(gi, oi):
            for gs, os_ in zip(gi["steps"], oi["steps"]):
                assert abs(gs.score - os_["ppl"]) <= 2e-3 * os_["ppl"]          # the score field carries ppl_j
                assert bool(gs.halt & 1) == os_["halt"]

        diverged = compare_runs(gpu, orc, lambda s: abs(s["ppl"] - thr) <= 1e-3 * thr, ppl_agree) is not None
        if not diverged:
            assert gpu["tokens"] == ref and gpu["sl_hist"] == orc["sl_hist"]
        if q == 0.5:
            assert len(gpu["sl_hist"]) > 2                                      # lookaheads do vary


# ---- full-size verification block, fused draft loop, reproducibility -----------------------------------

def test_verify_13b_full_depth_block_of_11():
    """The verification forward exactly as bench.py launches it: 40 layers of the 13B shape, block of
    11 tokens at ctx 512 and blocks of 1 and 8 tokens at ctx 1024 (the micro-benchmark's context), weights
    drawn on the device; the oracle gets the same bytes.  Then the dense prompt
    pass on the same model (the weights take a while to draw: one test for both)."""
    shape = W.CFG2_TARGET
    d = dev()
    w = W.make_weights(shape, 0, "bf16", device=d)
    gm = B.DiscoModel(shape, w, d)
    w_host = {k: v.cpu() for k, v in w.items()}
    del w
    torch.cuda.empty_cache()
    print("[parity] 13B full depth: weights on host", flush=True)
    om = O.Model(shape, w_host, kv_bf16=True, cache_upcast=False)
    am = torch.zeros(16, dtype=torch.int32, device=d)
    # block of 11 at ctx 512, and the verification micro-benchmark's context (1024) with blocks of 1 and 8
    for ctx, M in ((512, 11), (1024, 1), (1024, 8)):
        fill = W.make_kv_fill(shape, ctx, 2)
        gkv = B.DiscoKV(gm, ctx + 32, 16)
        gkv.fill(fill.to(d))
        ws = gm.workspace(16, ctx + 32)
        blk = W.make_tokens(41, M, shape.vocab).tolist()
        tb = torch.tensor(blk, dtype=torch.int32, device=d)
        lg = torch.empty(M, shape.vocab, dtype=torch.float32, device=d)
        B.disco_verify(gm, gkv, tb, M, am, lg, ws)
        torch.cuda.synchronize()
        lg2 = torch.empty_like(lg)
        B.disco_kv_rollback(gkv, ctx)
        B.disco_verify(gm, gkv, tb, M, am, lg2, ws)
        torch.cuda.synchronize()
        assert torch.equal(lg, lg2)                      # split reductions add in a fixed order
        okv = om.new_cache(ctx + 32)
        okv.fill(fill)
        ref = om.forward(blk, okv)
        check_logits(lg, ref, f"verify 13B x40 layers ctx {ctx} M {M}")
        check_argmax(am[:M].tolist(), ref, "13B full depth")
        n_flag = sum(1 for r in range(M) if O.top2_margin(ref[r]) < MARGIN)
        print(f"[parity] 13B full depth ctx {ctx}: {n_flag} of {M} rows flagged by the top-2 margin", flush=True)
        del gkv, ws, okv
    # The prompt pass at full depth.  Against the oracle on a prompt it can walk in seconds (48 tokens, then a
    # 4-token block that reads the cache the pass wrote), and, at the size bench.py --prefill times (512
    # tokens), as a property: the dense pass and the same prompt in blocks of 16 through the forward verified
    # above must leave caches that give the same logits for a later block.  With 40 layers of freshly
    # computed bf16 keys and values (no exact pre-filled entries) every path sits at 3e-3 .. 4e-3 from
    # the oracle and from the other path (neighbouring-bf16 roundings of K and V, amplified layer by layer):
    # inside the stated bar of 2e-2, above the 2e-3 regression bar of the shallow cases; held to 8e-3 here.
    deep_bar = 8e-3
    n0 = 48
    toks = W.make_prompt(1, 512 + 4, shape.vocab).to(torch.int32)
    tt = toks.to(d)
    kv0 = B.DiscoKV(gm, n0 + 32, 16)
    ws0 = gm.workspace(16, n0 + 32)
    print("[parity] 13B full depth: dense prompt pass of 48 tokens", flush=True)
    last = torch.empty(shape.vocab, dtype=torch.float32, device=d)
    B.disco_prefill(gm, kv0, tt, n0, last, gm.prefill_workspace(n0, n0 + 32))
    l4 = torch.empty(4, shape.vocab, dtype=torch.float32, device=d)
    B.disco_verify(gm, kv0, tt.data_ptr() + 4 * n0, 4, am, l4, ws0)
    torch.cuda.synchronize()
    okv0 = om.new_cache(n0 + 32)
    ref0 = om.forward(toks[:n0].tolist(), okv0)
    check_logits(last[None], ref0[-1:], "prompt pass 13B x40 layers n 48: last logits", tight=deep_bar)
    check_logits(l4, om.forward(toks[n0:n0 + 4].tolist(), okv0), "13B x40 layers: block after the prompt pass", tight=deep_bar)
    n = 512
    kv_a, kv_b = B.DiscoKV(gm, n + 32, 16), B.DiscoKV(gm, n + 32, 16)
    ws2 = gm.workspace(16, n + 32)
    print("[parity] 13B full depth: dense prompt pass of 512 tokens", flush=True)
    B.disco_prefill(gm, kv_a, tt, n, None, gm.prefill_workspace(n, n + 32))
    for i in range(0, n, 16):
        B.disco_verify(gm, kv_b, tt.data_ptr() + 4 * i, 16, am, None, ws2)
    la = torch.empty(4, shape.vocab, dtype=torch.float32, device=d)
    lb = torch.empty_like(la)
    B.disco_verify(gm, kv_a, tt.data_ptr() + 4 * n, 4, am, la, ws2)
    B.disco_verify(gm, kv_b, tt.data_ptr() + 4 * n, 4, am, lb, ws2)
    torch.cuda.synchronize()
    assert kv_a.len == kv_b.len == n + 4 and bool(torch.isfinite(la).all())
    worst = float((la - lb).abs().max()) / float(lb.abs().max())
    print(f"[parity] 13B full depth: dense vs block-wise prompt of 512, later block: max rel diff {worst:.3e}", flush=True)
    assert worst <= deep_bar


def test_draft_loop_equals_step_by_step_and_gates_after_halt():
    shape = W.scaled_shape(W.CFG1_DRAFT, vocab=4096)
    d = dev()
    w = W.make_weights(shape, 3, "bf16")
    clf_p = W.make_classifier(100)
    gm = B.DiscoModel(shape, w, d)
    clf = B.DiscoClf(clf_p, d)
    ctx, cap = 200, 7
    fill = W.make_kv_fill(shape, ctx, 2).to(d)
    ws = gm.workspace(16, ctx + 32)
    logits = torch.empty(shape.vocab, dtype=torch.float32, device=d)
    tok0 = torch.tensor([11, 12], dtype=torch.int32, device=d)

    # reference: one call per step with a host decision in between
    kv = B.DiscoKV(gm, ctx + 32, 16)
    kv.fill(fill)
    out = B.struct_tensor(B.ClfOut, 1, d)
    nxt = torch.zeros(1, dtype=torch.int32, device=d)
    scratch = B.classify_scratch(d)            # the loop uses the many-workgroup classify: so does the reference
    # scores grow with the block position under the seeded classifier: take tau between step 3 and 4
    B.disco_draft_step(gm, kv, tok0, 2, logits, ws)
    recs = []
    for j in range(1, cap + 1):
        B.disco_classify(clf, logits, shape.vocab, float(j), 0.0, 0, out, token_next=nxt, scratch=scratch)
        torch.cuda.synchronize()
        recs.append(B.read_struct(B.ClfOut, out))
        if j < cap:
            B.disco_draft_step(gm, kv, nxt, 1, logits, ws)
    ref_scores = [r.score for r in recs]
    assert all(b > a for a, b in zip(ref_scores, ref_scores[1:]))
    for tau, want_sl in ((0.0, cap), (2.0, 1)):
        kv2 = B.DiscoKV(gm, ctx + 32, 16)
        kv2.fill(fill)
        steps = B.struct_tensor(B.ClfOut, 16, d)
        lo_d = B.struct_tensor(B.LoopOut, 1, d)
        lo_h = B.struct_tensor(B.LoopOut, 1, pinned=True)
        B.disco_draft_loop(gm, kv2, clf, tok0, 2, cap, 0, 1.0, tau, None, logits, steps, lo_d, lo_h, ws)
        torch.cuda.synchronize()
        lo = B.LoopOut.from_buffer_copy(lo_h.numpy().tobytes())
        assert lo.sl == want_sl and lo.block[0] == 12
        assert kv2.len == ctx + 2 + cap - 1            # host length advanced for every enqueued step
        B.disco_kv_rollback(kv2, ctx + 2 + lo.sl - 1)
        got = [B.read_struct(B.ClfOut, steps, i) for i in range(cap)]
        for j in range(cap):
            if j < want_sl:
                assert got[j].executed == 1 and got[j].token == recs[j].token == lo.block[j + 1]
                assert list(got[j].feats) == list(recs[j].feats) and got[j].score == recs[j].score
                assert got[j].halt == (1 if j == want_sl - 1 else 0)
            else:
                assert got[j].executed == 0              # gated off on the device
    # static lookahead: exactly gamma steps whatever the classifier says
    kv3 = B.DiscoKV(gm, ctx + 32, 16)
    kv3.fill(fill)
    steps = B.struct_tensor(B.ClfOut, 16, d)
    lo_d = B.struct_tensor(B.LoopOut, 1, d)
    B.disco_draft_loop(gm, kv3, clf, tok0, 2, cap, 4, 1.0, 2.0, None, logits, steps, lo_d, None, ws)
    torch.cuda.synchronize()
    lo = B.read_struct(B.LoopOut, lo_d)
    assert lo.sl == 4 and list(lo.block[1:5]) == [r.token for r in recs[:4]]
    assert kv3.len == ctx + 2 + 4 - 1


# ---- more shapes and edges ----------------------------------------------------------------------------

def test_loop_mqa_pair_with_shared_embedding_table():
    """Multi-query LayerNorm/GELU pair (the code-model workload's structure, small): the draft reads
    the first d_draft columns of the target's embedding table through tok_emb_stride."""
    st = W.ModelShape("A", 2, 256, 2, 128, 1, 512, 496, max_pos=256)
    sd = W.ModelShape("A", 1, 128, 2, 64, 1, 256, 496, max_pos=256)
    tw = W.make_weights(st, 0, "bf16", sigma=0.08, gain_jitter=0.1)
    dw = W.make_weights(sd, 10, "bf16", sigma=0.08, gain_jitter=0.1)
    dw["tok_emb"] = tw["tok_emb"][:, :sd.d_model]              # oracle: a strided view of the same values
    ot, od = O.Model(st, tw, kv_bf16=True), O.Model(sd, dw, kv_bf16=True)
    clf = W.make_classifier(100)
    prompt = W.make_prompt(1, 50, st.vocab).tolist()
    n_new = 64
    ref, margins = O.greedy_target(ot, prompt, n_new)
    force = {"mask": W.make_force_mask(5, n_new, 0.6), "tokens": ref}
    d = dev()
    gt = B.DiscoModel(st, tw, d)
    gd = B.DiscoModel(sd, dw, d, tok_emb=gt.tok_emb, tok_emb_stride=st.d_model)
    eng = SpecEngine(gt, gd, B.DiscoClf(clf, d), max_ctx=140, page_tokens=8)
    for pol in ({"mode": "static", "gamma": 4}, {"mode": "disco", "tau": 0.6, "sl_max": 10, "pos_mode": "block"}):
        orc = O.spec_decode(ot, od, clf, prompt, n_new, pol, force=force)
        assert orc["tokens"] == ref
        gpu = eng.generate(prompt, n_new, pol, force=force, trace=True)
        if not _compare_runs(gpu, orc, pol.get("tau")):
            assert gpu["tokens"] == ref and gpu["sl_hist"] == orc["sl_hist"]


@pytest.mark.parametrize("hidden", [1, 37, 256])
def test_classifier_hidden_sizes(hidden):
    shape = W.ClassifierShape(hidden=hidden)
    clf = W.make_classifier(7, shape, sigma=0.5)
    g = torch.Generator().manual_seed(hidden)
    x = torch.randn(32000, generator=g) * 1.5
    for pos in (1.0, 40.0):
        r, _ = _run_classify(x, clf, pos, 0.5)
        f = O.features(x.double(), pos)
        c = O.classifier(f["feats"], clf)
        assert abs(r.score - c) < 2e-5, (hidden, pos, r.score, c)
        if abs(c - 0.5) > 1e-3:
            assert r.halt == int(c < 0.5)


def test_kv_capacity_and_page_edges():
    shape = SMALL_B_GQA
    om, gm, okv, gkv, ws = setup_pair(shape, 12, kv_ctx=40, page_tokens=8, permute=True, capacity=64)
    d = dev()
    am = torch.zeros(16, dtype=torch.int32, device=d)
    toks = W.make_tokens(9, 40, shape.vocab).tolist()

    def both(block, what):
        tb = torch.tensor(block, dtype=torch.int32, device=d)
        lg = torch.empty(len(block), shape.vocab, dtype=torch.float32, device=d)
        B.disco_verify(gm, gkv, tb, len(block), am, lg, ws)
        torch.cuda.synchronize()
        check_logits(lg, om.forward(block, okv), what)

    both(toks[:8], "fill to a page edge (48)")
    assert gkv.len == 48 and gkv.pages_in_use == 6
    both(toks[8:24], "fill to capacity (64)")
    assert gkv.len == 64 and gkv.pages_in_use == 8
    with pytest.raises(B.DiscoError) as e:                       # full: refused on the host, nothing launched
        B.disco_verify(gm, gkv, torch.tensor([1], dtype=torch.int32, device=d), 1, am, None, ws)
    assert e.value.code == B.ECAP and gkv.len == 64
    for new_len in (49, 48, 47):                                 # one past, on, one before a page edge
        B.disco_kv_rollback(gkv, new_len)
        okv.rollback(new_len)
        assert gkv.pages_in_use == (new_len + 7) // 8
        both(toks[24:24 + 5], f"after rollback to {new_len}")
        assert gkv.len == new_len + 5
