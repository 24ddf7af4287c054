"""CPU oracle for one DISCO speculative-decoding iteration and the generation loop around it.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, float64 statement of what the GPU path
must compute.  Only tests, the smoke check and the CPU-baseline leg of the benchmark may import
it; the product path never does, and this file imports nothing from the product.

Written from the paper (arXiv 2405.04304):
  * Sec. 2 (Background) and Fig. 1: a draft model generates SL tokens autoregressively, the target
    model checks all of them in one parallel forward, and accepts a prefix of them.
  * Sec. 3, "Finding the optimal SL per iteration": the oracle SL drafts until the first draft/target
    mismatch; mismatch is decided by rejection sampling at zero temperature, i.e. by comparing the
    draft token with the target's arg-max token.
  * Sec. 3, Eq. 2 and its footnote: C_i = FFN(Concat(Top_k(y_i), Ent(y_i), i)), k = 10; C_i is
    compared with a threshold tau; at most SL_max tokens are drafted per iteration.
  * Sec. 4 "SL classifier training": the FFN is a shallow two-layer network.
  * App. D.1: features are the top-k probabilities, the entropy, and the token position counted
    from the start of generation.
  * Sec. 3 (end) and App. F: the method keeps the rejection-sampling scheme of speculative decoding
    [Leviathan et al. 2023; Chen et al. 2023], which preserves the target's distribution, and is
    reported at temperature 1 as well: a draft token x drawn from the draft distribution q is kept
    with probability min(1, p(x) / q(x)) (p = target distribution at that position); at the first
    rejection a token is drawn from norm(max(0, p - q)); if every draft token is kept, a bonus
    token is drawn from the target's next distribution.
  * Sec. 4 "SL classifier training" and App. D.1: the classifier is trained with a cross-entropy
    loss on (features, accepted / rejected) pairs from a labelling run in which the draft predicts one
    token from the prompt plus the target's own continuation; its quality is reported as F1.
The two transformer families are not the paper's subject (it uses published checkpoints as black
boxes); their definitions below are the standard pre-norm decoder equations.

Readings of points the paper leaves open:
  the two rule-based baselines are named but not specified in the paper: the dynamic heuristic is
  taken as "lookahead + 2 after a fully accepted block, otherwise - 1 (not below 1), starting at 5";
  the perplexity rule as "stop when exp(-mean ln p) of the block's draft tokens exceeds a threshold";
  halt iff C_i < tau (strict); the token whose features triggered the halt stays in the block;
  entropy is over the full vocabulary in nats; features use the temperature-1 softmax of the raw
  draft logits; top-k values are in descending order; arg-max ties go to the lowest token id;
  position feature i counts generated tokens from 1 (mode "absolute") or restarts at 1 in every
  block (mode "block"); LayerNorm eps 1e-5, RMSNorm eps 1e-6, exact (erf) GELU, rotary base 10000
  with half-split pairing (c, c + d_head/2), no linear biases, untied LM head.
  Sampling (temperature > 0): distributions are softmax(logits / T); a token is drawn from a
  distribution by inverting its cumulative sum in vocabulary order at u * total, u uniform in
  [0, 1) and supplied by the caller (so oracle and GPU consume the same random numbers); the
  classifier's features stay those of the temperature-1 softmax of the raw draft logits.
  Training (the paper names only the loss): mean binary cross-entropy on the boolean labels,
  features standardised per component (mean, standard deviation of the training set), full-batch
  gradient descent with a fixed step for a fixed number of epochs from given initial parameters;
  the standardisation is folded into W1 and b1 afterwards, so the classifier keeps consuming raw
  features.  "Accepted" is predicted when C >= tau (the loop's continue condition).

Parity pins: every function here is pinned by tests/test_oracle_*.py (closed forms, library
routines, invariants, brute force); none is "parity unpinned".
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import torch

F64 = torch.float64


# --------------------------------------------------------------------------------------------
# building blocks
# --------------------------------------------------------------------------------------------

def layernorm(x: torch.Tensor, g: torch.Tensor, b: torch.Tensor, eps: float) -> torch.Tensor:
    """(x - mean) / sqrt(var + eps) * g + b over the last axis, biased variance."""
    mu = x.mean(dim=-1, keepdim=True)
    var = ((x - mu) ** 2).mean(dim=-1, keepdim=True)
    return (x - mu) / torch.sqrt(var + eps) * g + b


def rmsnorm(x: torch.Tensor, g: torch.Tensor, eps: float) -> torch.Tensor:
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    ms = (x ** 2).mean(dim=-1, keepdim=True)
    return x / torch.sqrt(ms + eps) * g


def gelu(x: torch.Tensor) -> torch.Tensor:
    """Exact GELU: x * Phi(x)."""
    return 0.5 * x * (1.0 + torch.erf(x / math.sqrt(2.0)))


def silu(x: torch.Tensor) -> torch.Tensor:
    return x / (1.0 + torch.exp(-x))


def rotary(x: torch.Tensor, pos: int, base: float) -> torch.Tensor:
    """Rotate x[..., d_head] at absolute position pos; pairs are (c, c + d_head/2)."""
    dh = x.shape[-1]
    half = dh // 2
    c = torch.arange(half, dtype=F64)
    ang = pos * base ** (-2.0 * c / dh)
    cs, sn = torch.cos(ang), torch.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return torch.cat([a * cs - b * sn, b * cs + a * sn], dim=-1)


def round_bf16(x: torch.Tensor) -> torch.Tensor:
    """Value of x after storage as bfloat16 (round to nearest even)."""
    return x.to(torch.float32).to(torch.bfloat16).to(F64)


class KVCache:
    """Keys and values of every layer for positions [0, len)."""

    def __init__(self, shape, capacity: int):
        self.k = torch.zeros(shape.n_layers, capacity, shape.n_kv_heads, shape.d_head, dtype=F64)
        self.v = torch.zeros_like(self.k)
        self.len = 0
        self.capacity = capacity

    def rollback(self, new_len: int) -> None:
        """Forget positions >= new_len (the rejected suffix of a draft block)."""
        if not 0 <= new_len <= self.len:
            raise ValueError("rollback target outside [0, len]")
        self.len = new_len

    def fill(self, kv: torch.Tensor) -> None:
        """Install given keys/values [n_layers, 2, ctx, n_kv, d_head] as positions [0, ctx)."""
        ctx = kv.shape[2]
        self.k[:, :ctx] = kv[:, 0].to(F64)
        self.v[:, :ctx] = kv[:, 1].to(F64)
        self.len = ctx


class Model:
    """Decoder-only transformer evaluated in float64 on the given (bf16- or fp32-valued) weights.

    kv_bf16: keys (after rotary) and values are rounded to bfloat16 when they enter the cache,
    because bf16 KV storage is part of the bf16 workloads' definition.
    """

    def __init__(self, shape, weights: Dict[str, torch.Tensor], kv_bf16: bool = False,
                 cache_upcast: Optional[bool] = None):
        self.shape = shape
        self.weights = weights
        self.kv_bf16 = kv_bf16
        if cache_upcast is None:
            cache_upcast = sum(w.numel() for w in weights.values()) < 300_000_000
        self._cache = {} if cache_upcast else None

    def w(self, name: str) -> torch.Tensor:
        if self._cache is None:
            return self.weights[name].to("cpu").to(F64)
        if name not in self._cache:
            self._cache[name] = self.weights[name].to("cpu").to(F64)
        return self._cache[name]

    def new_cache(self, capacity: int) -> KVCache:
        return KVCache(self.shape, capacity)

    def _norm(self, x, prefix):
        s = self.shape
        if s.family == "A":
            return layernorm(x, self.w(prefix + "_g"), self.w(prefix + "_b"), s.ln_eps)
        return rmsnorm(x, self.w(prefix + "_g"), s.rms_eps)

    def embed(self, tokens: Sequence[int], pos0: int) -> torch.Tensor:
        s = self.shape
        idx = torch.as_tensor(list(tokens), dtype=torch.long)
        h = self.weights["tok_emb"].to("cpu")[idx].to(F64)
        if s.family == "A":
            p = torch.arange(pos0, pos0 + len(idx))
            h = h + self.weights["pos_emb"].to("cpu")[p].to(F64)
        return h

    def attention(self, q: torch.Tensor, kv: KVCache, layer: int, pos0: int) -> torch.Tensor:
        """q [M, n_heads, d_head]; query j (absolute position pos0 + j) attends to cache positions
        0 .. pos0 + j inclusive.  Returns [M, n_heads * d_head]."""
        s = self.shape
        group = s.n_heads // s.n_kv_heads
        out = torch.zeros(q.shape[0], s.n_heads, s.d_head, dtype=F64)
        for j in range(q.shape[0]):
            n = pos0 + j + 1
            for hq in range(s.n_heads):
                hk = hq // group
                keys = kv.k[layer, :n, hk]                   # [n, d_head]
                vals = kv.v[layer, :n, hk]
                score = keys @ q[j, hq] / math.sqrt(s.d_head)
                p = torch.softmax(score, dim=0)
                out[j, hq] = p @ vals
        return out.reshape(q.shape[0], s.d_q)

    def forward(self, tokens: Sequence[int], kv: KVCache, return_hidden: bool = False):
        """Feed len(tokens) tokens at positions kv.len ..; append their keys/values; return the
        float64 logits [M, vocab] of every fed token (causal inside the block)."""
        s = self.shape
        m, pos0 = len(tokens), kv.len
        if pos0 + m > kv.capacity:
            raise ValueError("KV capacity exceeded")
        h = self.embed(tokens, pos0)
        for l in range(s.n_layers):
            p = f"l{l}."
            x = self._norm(h, p + "norm1")
            qkv = x @ self.w(p + "wqkv").T
            q = qkv[:, :s.d_q].reshape(m, s.n_heads, s.d_head)
            k = qkv[:, s.d_q:s.d_q + s.d_kv].reshape(m, s.n_kv_heads, s.d_head)
            v = qkv[:, s.d_q + s.d_kv:].reshape(m, s.n_kv_heads, s.d_head)
            if s.family == "B":
                q = torch.stack([rotary(q[j], pos0 + j, s.rope_base) for j in range(m)])
                k = torch.stack([rotary(k[j], pos0 + j, s.rope_base) for j in range(m)])
            if self.kv_bf16:
                k, v = round_bf16(k), round_bf16(v)
            kv.k[l, pos0:pos0 + m] = k
            kv.v[l, pos0:pos0 + m] = v
            h = h + self.attention(q, kv, l, pos0) @ self.w(p + "wo").T
            x = self._norm(h, p + "norm2")
            if s.family == "A":
                h = h + gelu(x @ self.w(p + "w1").T) @ self.w(p + "w2").T
            else:
                h = h + (silu(x @ self.w(p + "wg").T) * (x @ self.w(p + "wu").T)) @ self.w(p + "wd").T
        kv.len = pos0 + m
        logits = self._norm(h, "normf") @ self.w("wlm").T
        return (logits, h) if return_hidden else logits

    def prefill(self, tokens: Sequence[int], kv: KVCache, chunk: int = 64) -> None:
        for i in range(0, len(tokens), chunk):
            self.forward(tokens[i:i + chunk], kv)


# --------------------------------------------------------------------------------------------
# Eq. 2: features and classifier
# --------------------------------------------------------------------------------------------

def argmax_lowest(x: torch.Tensor) -> int:
    """Index of the maximum; the lowest index among equal maxima."""
    m = x.max()
    return int(torch.nonzero(x == m)[0, 0])


def top2_margin(x: torch.Tensor) -> float:
    t = torch.topk(x, 2).values
    return float(t[0] - t[1])


def features(logits: torch.Tensor, pos_feature: float, k: int = 10) -> Dict:
    """Top-k probabilities (descending), Shannon entropy in nats, and the position scalar, from the
    softmax of the raw logits.  Everything in float64; the feature vector is returned as the
    float32 values the classifier is fed."""
    x = logits.to(F64)
    m = x.max()
    e = torch.exp(x - m)
    p = e / e.sum()
    top = torch.sort(p, descending=True).values[:k]
    nz = p[p > 0]
    ent = float(-(nz * torch.log(nz)).sum())
    f = torch.cat([top, torch.tensor([ent, float(pos_feature)], dtype=F64)])
    return {"token": argmax_lowest(x), "feats": f.to(torch.float32), "probs": p,
            "margin": top2_margin(x)}


def classifier(feats: torch.Tensor, clf: Dict[str, torch.Tensor]) -> float:
    """C = sigmoid(w2 . relu(W1 f + b1) + b2), float64 arithmetic on float32 inputs."""
    f = feats.to(F64)
    hid = torch.relu(clf["W1"].to(F64) @ f + clf["b1"].to(F64))
    z = float(clf["w2"].to(F64) @ hid + clf["b2"].to(F64)[0])
    return 1.0 / (1.0 + math.exp(-z))


def accept(block: Sequence[int], target_argmax: Sequence[int]):
    """Greedy acceptance (rejection sampling at temperature 0, Fig. 1).

    block = [t_0, d_1 .. d_SL]; target_argmax[j] = the target's arg-max after seeing block[0..j].
    n = length of the longest prefix d_1..d_n with d_j == target_argmax[j-1]; the iteration emits
    d_1..d_n followed by target_argmax[n] (the correction, or the bonus token when n == SL)."""
    sl = len(block) - 1
    n = 0
    while n < sl and block[n + 1] == target_argmax[n]:
        n += 1
    return n, [int(t) for t in block[1:n + 1]] + [int(target_argmax[n])]


# --------------------------------------------------------------------------------------------
# sampling at temperature > 0: the rejection-sampling scheme the method keeps (Sec. 3, App. F)
# --------------------------------------------------------------------------------------------

def softmax_t(logits: torch.Tensor, temperature: float) -> torch.Tensor:
    """softmax(logits / T) in float64."""
    x = logits.to(F64) / float(temperature)
    e = torch.exp(x - x.max())
    return e / e.sum()


def sample_index(weights: torch.Tensor, u: float):
    """Draw from the distribution proportional to `weights` (non-negative, not necessarily
    normalised) by inverting its cumulative sum in index order: the smallest v with
    cumsum(weights)[v] > u * total.  Returns (v, margin) where margin is the distance, as a fraction
    of the total, between u * total and the nearest boundary of v's interval: a draw with a tiny
    margin is one that arithmetic in another precision may place in the neighbouring interval."""
    w = weights.to(F64)
    cdf = torch.cumsum(w, dim=0)
    total = float(cdf[-1])
    x = float(u) * total
    v = int(torch.searchsorted(cdf, torch.tensor(x, dtype=F64), right=True))
    pos = torch.nonzero(w > 0)
    last = int(pos[-1, 0])
    if v > last:                      # u * total landed on the end of the support
        v = last
    lo = float(cdf[v - 1]) if v > 0 else 0.0
    hi = float(cdf[v])
    margin = min(x - lo, hi - x) / total
    return v, margin


def accept_stochastic(block: Sequence[int], q_rows: Sequence[torch.Tensor], p_rows: Sequence[torch.Tensor],
                      u_accept: Sequence[float], u_resample: Sequence[float]):
    """Speculative sampling over one block.

    block = [t_0, d_1 .. d_SL]; q_rows[j-1] = the draft distribution d_j was drawn from;
    p_rows[j] = the target distribution after block[0..j] (j = 0..SL).  d_j is kept iff
    u_accept[j-1] < min(1, p_rows[j-1][d_j] / q_rows[j-1][d_j]).  At the first rejection (j = n + 1)
    the iteration's last token is drawn from norm(max(0, p_rows[n] - q_rows[n])); when all SL are
    kept it is drawn from p_rows[SL]; that draw uses u_resample[n].  Returns n, the emitted tokens,
    and per-decision margins."""
    sl = len(block) - 1
    n = 0
    acc_margins = []
    while n < sl:
        x = int(block[n + 1])
        p, q = float(p_rows[n][x]), float(q_rows[n][x])
        # u < min(1, p / q)  <=>  u * q < p  (u < 1 always)
        acc_margins.append(abs(float(u_accept[n]) * q - p) / max(q, 1e-300))
        if float(u_accept[n]) * q < p:
            n += 1
        else:
            break
    if n < sl:
        resid = torch.clamp(p_rows[n].to(F64) - q_rows[n].to(F64), min=0.0)
        last, smargin = sample_index(resid, float(u_resample[n]))
    else:
        last, smargin = sample_index(p_rows[sl], float(u_resample[n]))
    return n, [int(t) for t in block[1:n + 1]] + [last], {"accept_margins": acc_margins, "sample_margin": smargin}


# --------------------------------------------------------------------------------------------
# classifier training (Sec. 4 "SL classifier training", App. D.1)
# --------------------------------------------------------------------------------------------

def label_run(draft: Model, prompt: Sequence[int], reference: Sequence[int], force: Optional[Dict] = None,
              prefill_chunk: int = 64) -> Dict:
    """App. D.1: at every generated position the draft predicts ONE token from the prompt plus the
    target's own continuation (`reference`, the target's greedy text); the pair (Eq. 2 features of
    that prediction, draft token == target token) is one training example.  Position feature: 1 for
    the first generated token.  force: as in spec_decode."""
    kv = draft.new_cache(len(prompt) + len(reference) + 1)
    draft.prefill(list(prompt[:-1]), kv, prefill_chunk)
    feats, labels, margins = [], [], []
    last = int(prompt[-1])
    for p, ref_tok in enumerate(reference):
        logits = draft.forward([last], kv)[0].clone()
        if force is not None and bool(force["mask"][p]):
            logits[int(force["tokens"][p])] = logits.max() + 4.0
        ft = features(logits, p + 1)
        feats.append(ft["feats"])
        labels.append(int(ft["token"] == int(ref_tok)))
        margins.append(ft["margin"])
        last = int(ref_tok)
    return {"feats": torch.stack(feats), "labels": torch.tensor(labels, dtype=torch.int32), "margins": margins}


def _bce_with_logits(z: torch.Tensor, y: torch.Tensor) -> torch.Tensor:
    """-(y ln C + (1 - y) ln (1 - C)) with C = sigmoid(z), in the overflow-free form."""
    return torch.clamp(z, min=0.0) - z * y + torch.log1p(torch.exp(-z.abs()))


def clf_train(feats: torch.Tensor, labels: torch.Tensor, init: Dict[str, torch.Tensor], epochs: int, lr: float):
    """Train C = sigmoid(w2 . relu(W1 f + b1) + b2) on (features [N, 12], labels [N] in {0, 1}).

    Features are standardised, s = (f - mean) / max(std, 1e-6) (population standard deviation of the
    training set); the loss is the mean binary cross-entropy; every epoch takes one full-batch
    gradient step of size lr starting from `init` (read as parameters in the standardised space).
    Returns the parameters folded back to raw features, W1' = W1 / std, b1' = b1 - W1 (mean / std),
    and the loss before each step."""
    f = feats.to(F64)
    y = labels.to(F64)
    n = f.shape[0]
    mu = f.mean(dim=0)
    sd = torch.sqrt(((f - mu) ** 2).mean(dim=0)).clamp(min=1e-6)
    s = (f - mu) / sd
    W1, b1 = init["W1"].to(F64).clone(), init["b1"].to(F64).clone()
    w2, b2 = init["w2"].to(F64).clone(), init["b2"].to(F64).clone()
    losses = []
    for _ in range(epochs):
        a = s @ W1.T + b1                        # [N, hidden]
        act = torch.relu(a)
        z = act @ w2 + b2[0]
        losses.append(float(_bce_with_logits(z, y).mean()))
        dz = (torch.sigmoid(z) - y) / n          # d loss / d z
        g_w2 = act.T @ dz
        g_b2 = dz.sum()
        da = (dz[:, None] * w2[None, :]) * (a > 0).to(F64)
        g_W1 = da.T @ s
        g_b1 = da.sum(dim=0)
        W1 -= lr * g_W1; b1 -= lr * g_b1; w2 -= lr * g_w2; b2 -= lr * g_b2
    folded = {"W1": (W1 / sd).to(torch.float32), "b1": (b1 - (W1 * (mu / sd)).sum(dim=1)).to(torch.float32),
              "w2": w2.to(torch.float32), "b2": b2.to(torch.float32)}
    return folded, losses


def clf_eval(feats: torch.Tensor, labels: torch.Tensor, clf: Dict[str, torch.Tensor], tau: float) -> Dict:
    """Scores, confusion counts and F1 of the prediction "accepted iff C >= tau" (App. D.2)."""
    scores = [classifier(feats[i], clf) for i in range(feats.shape[0])]
    pred = [int(c >= tau) for c in scores]
    y = [int(v) for v in labels]
    tp = sum(1 for p_, t in zip(pred, y) if p_ and t)
    fp = sum(1 for p_, t in zip(pred, y) if p_ and not t)
    fn = sum(1 for p_, t in zip(pred, y) if not p_ and t)
    tn = len(y) - tp - fp - fn
    f1 = 2 * tp / (2 * tp + fp + fn) if (2 * tp + fp + fn) else 0.0
    return {"scores": scores, "tp": tp, "fp": fp, "fn": fn, "tn": tn, "f1": f1}


# --------------------------------------------------------------------------------------------
# generation loops
# --------------------------------------------------------------------------------------------

def greedy_target(target: Model, prompt: Sequence[int], max_new: int, prefill_chunk: int = 64):
    """Plain greedy decoding of the target: the definition of the text every policy must emit."""
    kv = target.new_cache(len(prompt) + max_new + 1)
    target.prefill(list(prompt[:-1]), kv, prefill_chunk)
    out, margins, last = [], [], int(prompt[-1])
    for _ in range(max_new):
        logits = target.forward([last], kv)[0]
        last = argmax_lowest(logits)
        out.append(last)
        margins.append(top2_margin(logits))
    return out, margins


def spec_decode(target: Model, draft: Model, clf: Optional[Dict], prompt: Sequence[int],
                max_new: int, policy: Dict, force: Optional[Dict] = None,
                prefill_chunk: int = 64) -> Dict:
    """Speculative decoding with a lookahead policy.

    policy: {"mode": "static", "gamma": g}
          | {"mode": "disco", "tau": t, "sl_max": c, "pos_mode": "absolute" | "block"}
          | {"mode": "oracle", "reference": greedy target tokens, "sl_max": optional cap}
          | {"mode": "heuristic", "start": s, "up": u, "down": d, "sl_max": c}   (the dynamic heuristic the
            paper compares with: the lookahead of the next iteration is SL + u after an iteration in which
            every drafted token was accepted, max(1, SL - d) otherwise)
          | {"mode": "ppl", "threshold": t, "sl_max": c}   (App. F's rule-based baseline: stop drafting
            when the perplexity of the block's draft tokens so far, exp(-mean ln p_draft(token)),
            exceeds t; the token that crosses the threshold stays in the block)
    force (synthetic acceptance): {"mask": bool per generated index, "tokens": the target's greedy
    tokens}; at a masked index the draft logit of the target's token is raised to max + 4 before
    the features are taken, so the draft agrees with the target there.

    Both models prefill prompt[:-1]; prompt[-1] plays t_0 of the first iteration.
    Returns tokens, counters, and a per-iteration / per-draft-step trace.
    """
    mode = policy["mode"]
    pos_mode = policy.get("pos_mode", "absolute")
    cap_policy = {"static": policy.get("gamma"), "disco": policy.get("sl_max"),
                  "oracle": policy.get("sl_max", 10 ** 9), "heuristic": policy.get("sl_max"),
                  "ppl": policy.get("sl_max")}[mode]
    heur_sl = int(policy.get("start", 5)) if mode == "heuristic" else None
    room = len(prompt) + max_new + (cap_policy if mode != "oracle" else max_new) + 2
    kv_t, kv_d = target.new_cache(room), draft.new_cache(room)
    target.prefill(list(prompt[:-1]), kv_t, prefill_chunk)
    draft.prefill(list(prompt[:-1]), kv_d, prefill_chunk)

    seq = [int(t) for t in prompt]
    n_prompt = len(seq)
    iters: List[Dict] = []
    n_draft_fwd = n_target_fwd = 0
    while len(seq) - n_prompt < max_new:
        emitted = len(seq) - n_prompt
        remaining = max_new - emitted
        cap = min(cap_policy, remaining - 1)
        if mode == "heuristic":
            cap = min(cap, heur_sl)
        # tokens the draft has not seen yet: 1 normally, 2 after a fully accepted block
        pending = seq[kv_d.len:]
        assert cap == 0 or 1 <= len(pending) <= 2
        block, steps = [seq[-1]], []
        j = 0
        nll = 0.0                                  # -sum ln p_draft(token) over the block so far
        while j < cap:
            j += 1
            logits = draft.forward(pending, kv_d)[-1].clone()
            n_draft_fwd += 1
            gen_index = emitted + j - 1            # 0-based index of the token being guessed
            forced = False
            if force is not None and bool(force["mask"][gen_index]):
                logits[int(force["tokens"][gen_index])] = logits.max() + 4.0
                forced = True
            i_feat = (emitted + j) if pos_mode == "absolute" else j
            ft = features(logits, i_feat)
            d = ft["token"]
            score = classifier(ft["feats"], clf) if clf is not None else float("nan")
            if mode == "oracle" and d != int(policy["reference"][gen_index]):
                # the mismatching token is not part of the block: oracle SL counts accepted tokens
                steps.append({"j": j, "token": d, "mismatch": True, "feats": ft["feats"],
                              "score": score, "margin": ft["margin"], "forced": forced,
                              "pos_feature": i_feat, "gen_index": gen_index})
                break
            block.append(d)
            pending = [d]
            nll -= math.log(max(float(ft["probs"][d]), 1e-300))
            ppl = math.exp(nll / j)
            if mode == "disco":
                halt = score < policy["tau"] or j == cap
            elif mode == "ppl":
                halt = ppl > policy["threshold"] or j == cap
            else:
                halt = j == cap
            steps.append({"j": j, "token": d, "feats": ft["feats"], "score": score, "ppl": ppl,
                          "halt": bool(halt), "margin": ft["margin"], "forced": forced,
                          "pos_feature": i_feat, "gen_index": gen_index})
            if halt:
                break
        sl = len(block) - 1
        ctx_t = kv_t.len
        logits_t = target.forward(block, kv_t)
        n_target_fwd += 1
        a = [argmax_lowest(logits_t[r]) for r in range(sl + 1)]
        n, emit = accept(block, a)
        emit = emit[:remaining]
        seq.extend(emit)
        kv_t.rollback(ctx_t + n + 1)
        kv_d.rollback(min(kv_d.len, ctx_t + n + 1))
        if mode == "heuristic" and sl > 0:
            heur_sl = (min(heur_sl + int(policy.get("up", 2)), cap_policy) if n == sl
                       else max(1, heur_sl - int(policy.get("down", 1))))
        iters.append({"sl": sl, "n": n, "block": block, "target_argmax": a, "emit": emit,
                      "steps": steps, "ctx": ctx_t,
                      "target_margins": [top2_margin(logits_t[r]) for r in range(sl + 1)]})
    return {"tokens": seq[n_prompt:], "iterations": iters, "n_iterations": len(iters),
            "n_draft_forwards": n_draft_fwd, "n_target_forwards": n_target_fwd,
            "sl_hist": _hist([it["sl"] for it in iters])}


def spec_decode_sampling(target: Model, draft: Model, clf: Optional[Dict], prompt: Sequence[int],
                         max_new: int, policy: Dict, temperature: float, uniforms: Dict,
                         prefill_chunk: int = 64) -> Dict:
    """Speculative decoding at temperature > 0 with a lookahead policy ("static" or "disco").

    uniforms: {"draft": [max_new + cap] floats, one per generated index (the draw of the draft token
    guessed for that index), "accept": the same shape (the keep / reject draw for that index),
    "resample": the same shape, indexed by the generated index of the iteration's last token}.
    Indexing by generated position makes the random numbers a function of the position alone, as
    the forcing mask of the greedy workloads is.  The classifier's features come from the
    temperature-1 softmax of the raw draft logits; its position feature as in spec_decode."""
    mode = policy["mode"]
    assert mode in ("static", "disco")
    pos_mode = policy.get("pos_mode", "absolute")
    cap_policy = policy["gamma"] if mode == "static" else policy["sl_max"]
    room = len(prompt) + max_new + cap_policy + 2
    kv_t, kv_d = target.new_cache(room), draft.new_cache(room)
    target.prefill(list(prompt[:-1]), kv_t, prefill_chunk)
    draft.prefill(list(prompt[:-1]), kv_d, prefill_chunk)
    seq = [int(t) for t in prompt]
    n_prompt = len(seq)
    iters: List[Dict] = []
    while len(seq) - n_prompt < max_new:
        emitted = len(seq) - n_prompt
        remaining = max_new - emitted
        cap = min(cap_policy, remaining - 1)
        pending = seq[kv_d.len:]
        block, q_rows, steps = [seq[-1]], [], []
        j = 0
        while j < cap:
            j += 1
            logits = draft.forward(pending, kv_d)[-1]
            gen_index = emitted + j - 1
            q = softmax_t(logits, temperature)
            d, dmargin = sample_index(q, float(uniforms["draft"][gen_index]))
            i_feat = (emitted + j) if pos_mode == "absolute" else j
            ft = features(logits, i_feat)
            score = classifier(ft["feats"], clf) if clf is not None else float("nan")
            block.append(d)
            q_rows.append(q)
            pending = [d]
            halt = (j == cap) if mode == "static" else (score < policy["tau"] or j == cap)
            steps.append({"j": j, "token": d, "score": score, "halt": bool(halt), "sample_margin": dmargin,
                          "pos_feature": i_feat, "gen_index": gen_index, "feats": ft["feats"]})
            if halt:
                break
        sl = len(block) - 1
        ctx_t = kv_t.len
        logits_t = target.forward(block, kv_t)
        p_rows = [softmax_t(logits_t[r], temperature) for r in range(sl + 1)]
        u_acc = [float(uniforms["accept"][emitted + r]) for r in range(sl)]
        u_res = [float(uniforms["resample"][emitted + r]) for r in range(sl + 1)]
        n, emit, info = accept_stochastic(block, q_rows, p_rows, u_acc, u_res)
        emit = emit[:remaining]
        seq.extend(emit)
        kv_t.rollback(ctx_t + n + 1)
        kv_d.rollback(min(kv_d.len, ctx_t + n + 1))
        iters.append({"sl": sl, "n": n, "block": block, "emit": emit, "steps": steps, "ctx": ctx_t, **info})
    return {"tokens": seq[n_prompt:], "iterations": iters, "n_iterations": len(iters),
            "sl_hist": _hist([it["sl"] for it in iters])}


def _hist(xs: Sequence[int]) -> Dict[int, int]:
    h: Dict[int, int] = {}
    for x in xs:
        h[x] = h.get(x, 0) + 1
    return dict(sorted(h.items()))


def improvement_factor(alpha: float, gamma: int, c: float) -> float:
    """Eq. 1: expected speedup of static lookahead gamma at i.i.d. acceptance rate alpha and
    draft/target cost ratio c."""
    return (1.0 - alpha ** (gamma + 1)) / ((1.0 - alpha) * (gamma * c + 1.0))


def normalized_index(n_iterations: int) -> List[float]:
    """App. A: iteration k of a prompt with n iterations sits at k / (n - 1) on [0, 1]."""
    if n_iterations == 1:
        return [0.0]
    return [k / (n_iterations - 1) for k in range(n_iterations)]
