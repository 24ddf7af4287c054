"""Pins for the oracle's building blocks: library routines, closed forms, hand-worked cases.

None of these tests re-types the oracle's own formula: each compares against a PyTorch library
routine, a closed form, or an independently formulated computation (complex-number rotary,
full-sequence masked attention)."""
import math

import pytest
import torch
import torch.nn.functional as F

from oracle import disco_oracle as O
from workloads import synth as W

F64 = torch.float64
torch.manual_seed(1234)


# ---- textbook layers vs library routines -----------------------------------------------------

def test_layernorm_matches_library():
    x = torch.randn(5, 96, dtype=F64) * 3 + 0.7
    g, b = torch.randn(96, dtype=F64), torch.randn(96, dtype=F64)
    ref = F.layer_norm(x, (96,), g, b, eps=1e-5)
    assert torch.allclose(O.layernorm(x, g, b, 1e-5), ref, atol=1e-12)


def test_rmsnorm_matches_library():
    x = torch.randn(5, 96, dtype=F64) * 2 + 0.3
    g = torch.randn(96, dtype=F64)
    ref = F.rms_norm(x, (96,), g, eps=1e-6)
    assert torch.allclose(O.rmsnorm(x, g, 1e-6), ref, atol=1e-12)


def test_gelu_is_exact_erf_form_and_silu():
    x = torch.linspace(-6, 6, 101, dtype=F64)
    assert torch.allclose(O.gelu(x), F.gelu(x, approximate="none"), atol=1e-14)
    # the tanh approximation differs by up to ~5e-4: make sure that is not what we have
    assert (O.gelu(x) - F.gelu(x, approximate="tanh")).abs().max() > 1e-4
    assert torch.allclose(O.silu(x), F.silu(x), atol=1e-14)


def test_rotary_hand_case_and_invariants():
    # d_head = 2: one pair, frequency 1, so position p rotates (1, 0) to (cos p, sin p)
    r = O.rotary(torch.tensor([1.0, 0.0], dtype=F64), 3, 10000.0)
    assert torch.allclose(r, torch.tensor([math.cos(3.0), math.sin(3.0)], dtype=F64), atol=1e-15)
    # complex-number formulation with half-split pairing, frequencies base^(-2c/d)
    dh, base = 16, 10000.0
    x = torch.randn(3, dh, dtype=F64)
    for pos in (0, 1, 17, 2047):
        z = torch.complex(x[:, :dh // 2], x[:, dh // 2:])
        theta = torch.tensor([pos * base ** (-(2 * c) / dh) for c in range(dh // 2)], dtype=F64)
        zr = z * torch.polar(torch.ones_like(theta), theta)
        ref = torch.cat([zr.real, zr.imag], dim=-1)
        assert torch.allclose(O.rotary(x, pos, base), ref, atol=1e-12)
    # relative-position property: <rot(q,a), rot(k,b)> depends only on a - b
    q, k = torch.randn(dh, dtype=F64), torch.randn(dh, dtype=F64)
    d1 = O.rotary(q, 40, base) @ O.rotary(k, 33, base)
    d2 = O.rotary(q, 1007, base) @ O.rotary(k, 1000, base)
    assert abs(float(d1 - d2)) < 1e-10
    assert abs(float(O.rotary(q, 99, base).norm() - q.norm())) < 1e-12


def test_round_bf16_is_rne_on_8_bit_mantissa():
    # 1 + 2^-8 is exactly half-way between bf16 neighbours 1 and 1 + 2^-7: ties go to even (1.0)
    assert float(O.round_bf16(torch.tensor([1.0 + 2 ** -8], dtype=F64))) == 1.0
    assert float(O.round_bf16(torch.tensor([1.0 + 3 * 2 ** -8], dtype=F64))) == 1.0 + 2 ** -6
    assert float(O.round_bf16(torch.tensor([1.0 + 2 ** -8 + 2 ** -12], dtype=F64))) == 1.0 + 2 ** -7


# ---- whole forward vs an independent full-sequence implementation on library routines --------

def _reference_forward(shape, w, tokens):
    """No cache, whole sequence at once; attention via scaled_dot_product_attention(is_causal)."""
    T = len(tokens)
    d = {k: v.to(F64) for k, v in w.items()}
    h = d["tok_emb"][torch.tensor(tokens)]
    if shape.family == "A":
        h = h + d["pos_emb"][:T]

    def norm(x, p):
        if shape.family == "A":
            return F.layer_norm(x, (shape.d_model,), d[p + "_g"], d[p + "_b"], eps=shape.ln_eps)
        return F.rms_norm(x, (shape.d_model,), d[p + "_g"], eps=shape.rms_eps)

    def rope(x):  # x [T, H, dh] -> complex rotation
        dh = shape.d_head
        z = torch.complex(x[..., :dh // 2], x[..., dh // 2:])
        inv = shape.rope_base ** (-torch.arange(0, dh, 2, dtype=F64) / dh)
        ang = torch.arange(T, dtype=F64)[:, None] * inv[None, :]
        z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(shape.n_layers):
        p = f"l{l}."
        x = norm(h, p + "norm1")
        qkv = F.linear(x, d[p + "wqkv"])
        q = qkv[:, :shape.d_q].view(T, shape.n_heads, shape.d_head)
        k = qkv[:, shape.d_q:shape.d_q + shape.d_kv].view(T, shape.n_kv_heads, shape.d_head)
        v = qkv[:, shape.d_q + shape.d_kv:].view(T, shape.n_kv_heads, shape.d_head)
        if shape.family == "B":
            q, k = rope(q), rope(k)
        rep = shape.n_heads // shape.n_kv_heads
        k = k.repeat_interleave(rep, dim=1)
        v = v.repeat_interleave(rep, dim=1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1),
                                           v.transpose(0, 1), is_causal=True)
        h = h + F.linear(a.transpose(0, 1).reshape(T, shape.d_q), d[p + "wo"])
        x = norm(h, p + "norm2")
        if shape.family == "A":
            h = h + F.linear(F.gelu(F.linear(x, d[p + "w1"])), d[p + "w2"])
        else:
            h = h + F.linear(F.silu(F.linear(x, d[p + "wg"])) * F.linear(x, d[p + "wu"]), d[p + "wd"])
    return F.linear(norm(h, "normf"), d["wlm"])


SHAPES = {
    "A_mha": W.ModelShape("A", 2, 64, 4, 16, 4, 128, 97, max_pos=64),
    "A_mqa": W.ModelShape("A", 2, 64, 4, 16, 1, 128, 97, max_pos=64),
    "B_mha": W.ModelShape("B", 2, 64, 4, 16, 4, 96, 97),
    "B_gqa": W.ModelShape("B", 2, 64, 4, 16, 2, 96, 97),
}


@pytest.mark.parametrize("name", list(SHAPES))
def test_forward_matches_library_full_sequence(name):
    shape = SHAPES[name]
    # sigma 0.2 and jittered gains/biases so every term matters at the 1e-9 level
    w = W.make_weights(shape, seed=7, dtype="f32", sigma=0.2, gain_jitter=0.3)
    tokens = W.make_tokens(3, 19, shape.vocab).tolist()
    ref = _reference_forward(shape, w, tokens)
    m = O.Model(shape, w)
    kv = m.new_cache(32)
    got = m.forward(tokens, kv)                       # one 19-token block
    assert torch.allclose(got, ref, atol=1e-9, rtol=0)
    kv1 = m.new_cache(32)                             # token by token through the KV cache
    got1 = torch.cat([m.forward([t], kv1) for t in tokens])
    assert torch.allclose(got1, ref, atol=1e-9, rtol=0)
    kv2 = m.new_cache(32)                             # ragged chunks 7 + 1 + 11
    got2 = torch.cat([m.forward(tokens[:7], kv2), m.forward(tokens[7:8], kv2),
                      m.forward(tokens[8:], kv2)])
    assert torch.allclose(got2, ref, atol=1e-9, rtol=0)
    assert kv.len == kv1.len == kv2.len == 19


def test_block_is_causal_and_rollback_restores_state():
    shape = SHAPES["B_gqa"]
    w = W.make_weights(shape, seed=8, dtype="f32", sigma=0.2)
    m = O.Model(shape, w)
    ctx = W.make_tokens(4, 9, shape.vocab).tolist()
    blk_a, blk_b = [5, 6, 7, 8, 9], [5, 6, 70, 80, 90]
    kv = m.new_cache(32)
    m.forward(ctx, kv)
    la = m.forward(blk_a, kv)
    assert kv.len == 14
    kv.rollback(9)
    lb = m.forward(blk_b, kv)
    # rows 0,1 see identical prefixes; row 2 onwards sees a changed token
    assert torch.equal(la[:2], lb[:2])
    assert not torch.allclose(la[2], lb[2])
    fresh = m.new_cache(32)
    m.forward(ctx, fresh)
    assert torch.equal(m.forward(blk_b, fresh), lb)   # stale suffix left by block A is dead
    kv.rollback(kv.len)                               # no-op
    assert kv.len == 14
    with pytest.raises(ValueError):
        kv.rollback(15)
    with pytest.raises(ValueError):
        kv.rollback(-1)


def test_kv_bf16_stores_bf16_values_only():
    shape = SHAPES["B_mha"]
    w = W.make_weights(shape, seed=9, dtype="bf16", sigma=0.2)
    m = O.Model(shape, w, kv_bf16=True)
    kv = m.new_cache(16)
    m.forward([1, 2, 3], kv)
    k = kv.k[:, :3]
    assert torch.equal(k, k.to(torch.bfloat16).to(F64))
    m2 = O.Model(shape, w, kv_bf16=False)
    kv2 = m2.new_cache(16)
    m2.forward([1, 2, 3], kv2)
    assert not torch.equal(kv2.k[:, :3], k)
    # layer 0 sees identical inputs either way, so its keys differ by the bf16 rounding alone
    assert torch.allclose(kv2.k[0, :3], k[0], rtol=2 ** -8, atol=1e-30)


# ---- Eq. 2 features: closed forms -------------------------------------------------------------

def test_features_uniform_logits():
    V = 1000
    f = O.features(torch.full((V,), 3.25, dtype=F64), 7)
    assert f["token"] == 0                              # ties -> lowest id
    assert torch.allclose(f["feats"][:10], torch.full((10,), 1.0 / V), atol=1e-9)
    assert abs(float(f["feats"][10]) - math.log(V)) < 1e-6
    assert float(f["feats"][11]) == 7.0


def test_features_one_hot_spike_closed_form():
    V, L, at = 4097, 5.0, 1234
    x = torch.zeros(V, dtype=F64)
    x[at] = L
    f = O.features(x, 3)
    z = math.exp(L) + V - 1
    p1, pr = math.exp(L) / z, 1.0 / z
    H = -(p1 * math.log(p1) + (V - 1) * pr * math.log(pr))
    assert f["token"] == at
    assert abs(float(f["feats"][0]) - p1) < 1e-7
    assert torch.allclose(f["feats"][1:10], torch.full((9,), pr), atol=1e-9)
    assert abs(float(f["feats"][10]) - H) < 1e-6
    assert abs(f["margin"] - L) < 1e-12


def test_features_invariants_and_known_topk():
    g = torch.Generator().manual_seed(5)
    for V in (11, 64, 4096, 32000, 49152, 1001):
        x = torch.randn(V, generator=g, dtype=F64) * 2.0
        f = O.features(x, 1)
        f2 = O.features(x + 123.456, 1)                # shift invariance
        assert f2["token"] == f["token"]
        assert torch.allclose(f2["feats"], f["feats"], atol=1e-6)
        top, ent = f["feats"][:10].to(F64), float(f["feats"][10])
        assert (top[:-1] >= top[1:]).all() and float(top.sum()) <= 1 + 1e-6
        assert 0 <= ent <= math.log(V) + 1e-6 and ent >= -math.log(float(top[0])) - 1e-6
        ref = torch.softmax(x, 0)
        assert torch.allclose(top, torch.topk(ref, 10).values.to(torch.float32).to(F64), atol=1e-7)
        assert abs(ent - float(torch.distributions.Categorical(probs=ref).entropy())) < 1e-5
    # a permutation of known values: probabilities proportional to 2^k
    vals = torch.log(torch.tensor([2.0 ** k for k in range(12)], dtype=F64))
    perm = torch.randperm(12, generator=g)
    f = O.features(vals[perm], 0)
    want = torch.tensor([2.0 ** k for k in range(11, 1, -1)], dtype=F64) / (2.0 ** 12 - 1)
    assert torch.allclose(f["feats"][:10].to(F64), want, atol=1e-7)
    assert f["token"] == int(torch.nonzero(perm == 11)[0, 0])


def test_features_extreme_logits_do_not_overflow():
    x = torch.tensor([1000.0, 0.0, -1000.0], dtype=F64)
    f = O.features(x, 0, k=3)
    assert float(f["feats"][0]) == 1.0 and float(f["feats"][3]) == 0.0


# ---- classifier --------------------------------------------------------------------------------

def test_classifier_hand_example_and_zero_weights():
    # 12 -> 2 -> 1 by hand: hidden = relu([f0 + f10 - 1, -f11]) ; z = 2*h0 - 3*h1 + 0.5
    W1 = torch.zeros(2, 12)
    W1[0, 0], W1[0, 10], W1[1, 11] = 1.0, 1.0, -1.0
    clf = {"W1": W1, "b1": torch.tensor([-1.0, 0.0]), "w2": torch.tensor([2.0, -3.0]),
           "b2": torch.tensor([0.5])}
    f = torch.zeros(12)
    f[0], f[10], f[11] = 0.75, 1.5, 4.0
    z = 2.0 * (0.75 + 1.5 - 1.0) + 0.5                # second hidden unit is clipped by ReLU
    assert abs(O.classifier(f, clf) - 1 / (1 + math.exp(-z))) < 1e-12
    f[11] = -4.0                                       # now it is active: z -= 3 * 4
    assert abs(O.classifier(f, clf) - 1 / (1 + math.exp(-(z - 12.0)))) < 1e-12
    zero = {"W1": torch.zeros(64, 12), "b1": torch.zeros(64), "w2": torch.zeros(64),
            "b2": torch.zeros(1)}
    assert O.classifier(torch.randn(12), zero) == 0.5


def test_classifier_monotone_in_a_feature_with_positive_path():
    clf = {"W1": torch.eye(12)[:3], "b1": torch.zeros(3), "w2": torch.tensor([1.0, 0.0, 0.0]),
           "b2": torch.zeros(1)}
    scores = [O.classifier(torch.tensor([t] + [0.0] * 11), clf) for t in (-1.0, 0.0, 0.5, 2.0)]
    assert scores[0] == scores[1] == 0.5 and scores[1] < scores[2] < scores[3]


# ---- acceptance ---------------------------------------------------------------------------------

def _golden(name):
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    return [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]


def test_accept_fig1_example():
    (sl, n_acc), = [(int(a), int(b)) for a, b in _golden("fig1_accept.txt")]
    block = [100, 1, 2, 3, 4, 5]                       # t0, t1..t5
    target = [1, 2, 3, 40, 50, 60]                     # target agrees on t1..t3 only
    n, emit = O.accept(block, target)
    assert len(block) - 1 == sl and n == n_acc
    assert emit == [1, 2, 3, 40]                       # three accepted + the target's correction


def test_accept_edge_cases():
    assert O.accept([9], [4]) == (0, [4])                              # SL = 0: plain target step
    assert O.accept([9, 1, 2], [7, 2, 3]) == (0, [7])                  # first token rejected
    assert O.accept([9, 1, 2], [1, 2, 3]) == (2, [1, 2, 3])            # all accepted + bonus
    assert O.accept([9, 1, 2, 3], [1, 5, 3, 4]) == (1, [1, 5])         # later match is irrelevant


def test_normalized_index_appendix_example():
    rows = _golden("appA_normalized_index.txt")
    sls, want = [int(v) for v in rows[0]], [float(v) for v in rows[1]]
    assert O.normalized_index(len(sls)) == want
    assert O.normalized_index(1) == [0.0]
