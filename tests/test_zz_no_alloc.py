"""The classify call that allocates nothing (disco_classify_static: the many-workgroup reduction runs on
an array inside the library's code object) against disco_classify with a caller-supplied scratch buffer.
Both run the same kernels over the same launch shape, so the records must agree to the parity bar of
the classify tests: token and halt bit identical, features and score within fp32 rounding (here they are
bitwise equal).  Two calls in a row on the shared array, the second with a smaller vocabulary; then a
gated call and the size limit."""
import ctypes as C

import pytest
import torch

from paper_2405_04304_amd import binding as B
from workloads import synth as W

pytestmark = pytest.mark.gpu


def _record(t):
    r = B.read_struct(B.ClfOut, t)
    return r.token, list(r.feats), r.score, r.halt, r.executed


def test_classify_static_equals_classify_with_scratch():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    dev = torch.device("cuda:0")
    clf = B.DiscoClf(W.make_classifier(100), dev)
    scratch = B.classify_scratch(dev)
    g = torch.Generator().manual_seed(41)
    # every size takes the many-workgroup path (vocab >= 4096); the second and third are smaller than the
    # one before, so the array still holds records of the larger call
    for V, pos, force in ((49152, 3.0, None), (32000, 7.0, 1234), (4096, 1.0, None), (65536, 2.0, 65535)):
        x = (torch.randn(V, generator=g) * 1.7).to(torch.float32)
        outs = []
        for static in (False, True):
            xd = x.to(dev).clone()
            out = B.struct_tensor(B.ClfOut, 1, dev)
            nxt = torch.full((1,), -5, dtype=torch.int32, device=dev)
            cnt = torch.zeros(2, dtype=torch.int32, device=dev)
            ft = torch.tensor([force], dtype=torch.int32, device=dev) if force is not None else None
            print(f"[no-alloc] vocab {V} static {static}", flush=True)
            if static:
                B.disco_classify_static(clf, xd, V, pos, 0.5, 0, out, token_next=nxt, sl_count=cnt, force_token=ft)
            else:
                B.disco_classify(clf, xd, V, pos, 0.5, 0, out, token_next=nxt, sl_count=cnt, force_token=ft,
                                 scratch=scratch)
            torch.cuda.synchronize()
            outs.append((_record(out), int(nxt[0]), int(cnt[0]), xd.cpu()))
        (ra, na, ca, xa), (rb, nb, cb, xb) = outs
        assert ra[4] == 1 and rb[4] == 1
        assert ra[0] == rb[0] and na == nb == ra[0] and ca == cb == 1, (V, ra, rb)
        assert ra[3] == rb[3]
        assert torch.allclose(torch.tensor(ra[1]), torch.tensor(rb[1]), rtol=2e-5, atol=1e-6), (V, ra[1], rb[1])
        assert ra[1] == rb[1] and ra[2] == rb[2], "same kernels, same launch shape: bitwise equal"
        assert torch.equal(xa, xb)
        if force is not None:
            assert ra[0] == force


def test_classify_static_gate_and_limit():
    dev = torch.device("cuda:0")
    clf = B.DiscoClf(W.make_classifier(100), dev)
    x = torch.randn(32000, generator=torch.Generator().manual_seed(5)).to(dev)
    out = B.struct_tensor(B.ClfOut, 1, dev)
    gate = torch.ones(1, dtype=torch.int32, device=dev)
    B.disco_classify_static(clf, x, 32000, 1.0, 0.5, 0, out, gate=gate)
    torch.cuda.synchronize()
    assert B.read_struct(B.ClfOut, out).executed == 0
    gate.zero_()
    B.disco_classify_static(clf, x, 32000, 1.0, 0.5, 1, out, gate=gate)      # force_halt closes the gate
    torch.cuda.synchronize()
    assert B.read_struct(B.ClfOut, out).executed == 1 and int(gate[0]) == 1
    with pytest.raises(B.DiscoError) as e:
        B.disco_classify_static(clf, x, 65537, 1.0, 0.5, 0, out)
    assert e.value.code == B.ECAP
