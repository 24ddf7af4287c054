"""Host driver of the speculative-decoding loop over the C entry points.

One iteration = disco_draft_loop (draft steps + Eq. 2 classifier, no host round trip between steps)
-> disco_verify -> disco_accept -> disco_kv_rollback on both caches.  The host synchronises twice
per iteration: once to learn SL (it sizes the verification block) and once to learn the accepted
length.  This module moves token ids and lengths around; all arithmetic runs in the library."""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


class SpecEngine:
    def __init__(self, target: B.DiscoModel, draft: Optional[B.DiscoModel], clf: Optional[B.DiscoClf],
                 max_ctx: int, page_tokens: int = 16, page_order_target=None, page_order_draft=None):
        self.target, self.draft, self.clf = target, draft, clf
        self.dev = target.device
        self.max_ctx = max_ctx
        cap = max_ctx + B.MAX_BLOCK
        self.kv_t = B.DiscoKV(target, cap, page_tokens, page_order_target)
        self.ws_t = target.workspace(B.MAX_BLOCK, cap)
        if draft is not None:
            self.kv_d = B.DiscoKV(draft, cap, page_tokens, page_order_draft)
            self.ws_d = draft.workspace(B.MAX_BLOCK, cap)
            self.logits_d = torch.empty(draft.shape.vocab, dtype=torch.float32, device=self.dev)
        self.steps = B.struct_tensor(B.ClfOut, B.MAX_BLOCK, self.dev)
        self.loop_dev = B.struct_tensor(B.LoopOut, 1, self.dev)
        self.loop_host = B.struct_tensor(B.LoopOut, 1, pinned=True)
        self.acc_dev = B.struct_tensor(B.AcceptOut, 1, self.dev)
        self.acc_host = B.struct_tensor(B.AcceptOut, 1, pinned=True)
        self.argmax = torch.zeros(B.MAX_BLOCK, dtype=torch.int32, device=self.dev)
        self.tok_in = torch.zeros(B.MAX_BLOCK, dtype=torch.int32, device=self.dev)
        self.tok_stage = torch.zeros(B.MAX_BLOCK, dtype=torch.int32, pin_memory=True)

    # -- helpers ---------------------------------------------------------------------------------
    def _put_tokens(self, toks: Sequence[int]) -> None:
        n = len(toks)
        self.tok_stage[:n] = torch.as_tensor(list(toks), dtype=torch.int32)
        self.tok_in[:n].copy_(self.tok_stage[:n], non_blocking=True)

    def reset(self) -> None:
        B.disco_kv_rollback(self.kv_t, 0)
        if self.draft is not None:
            B.disco_kv_rollback(self.kv_d, 0)

    def prefill(self, tokens: Sequence[int], dense: Optional[bool] = None) -> None:
        """Feed the prompt through both models: one dense pass per model (32 tokens or more), otherwise
        blocks of DISCO_MAX_BLOCK tokens through the verification forward.  dense=True / False forces one
        of the two."""
        toks = torch.as_tensor(list(tokens), dtype=torch.int32).to(self.dev)
        n_all = len(tokens)
        for model, kv, ws in ((self.target, self.kv_t, self.ws_t),) + (
                ((self.draft, self.kv_d, self.ws_d),) if self.draft is not None else ()):
            use_dense = dense if dense is not None else n_all >= 32
            if use_dense and n_all > 0:
                for i in range(0, n_all, B.PREFILL_MAX):
                    n = min(B.PREFILL_MAX, n_all - i)
                    pws = model.prefill_workspace(n, kv.len + n + 16)
                    B.disco_prefill(model, kv, toks.data_ptr() + 4 * i, n, None, pws)
                    torch.cuda.synchronize(self.dev)         # the workspace is released after the pass
                    del pws
                continue
            for i in range(0, n_all, B.MAX_BLOCK):
                n = min(B.MAX_BLOCK, n_all - i)
                B.disco_verify(model, kv, toks.data_ptr() + 4 * i, n, self.argmax, None, ws)
        torch.cuda.synchronize(self.dev)

    def greedy(self, prompt: Sequence[int], max_new: int, progress=None) -> List[int]:
        """Plain greedy decoding of the target (verification blocks of one token)."""
        self.reset()
        self.prefill(prompt[:-1])
        out, last = [], int(prompt[-1])
        for i in range(max_new):
            if progress is not None and i % 32 == 0:
                progress(i)
            self._put_tokens([last])
            B.disco_verify(self.target, self.kv_t, self.tok_in, 1, self.argmax, None, self.ws_t)
            last = int(self.argmax[0].item())
            out.append(last)
        return out

    # -- labelling run and classifier training (App. D.1, Sec. 4) ---------------------------------
    def label_run(self, prompt: Sequence[int], reference: Sequence[int], force: Optional[Dict] = None):
        """At every generated position the draft predicts one token from the prompt plus the target's
        own continuation `reference`.  Returns device tensors: features [N, 12] (as disco_classify
        records them, position feature 1, 2, ...), labels [N] int32 (draft token == reference token),
        and the draft tokens."""
        n = len(reference)
        self.reset()
        self.prefill(prompt[:-1])
        fed = torch.as_tensor([int(prompt[-1])] + [int(t) for t in reference[:-1]], dtype=torch.int32).to(self.dev)
        ref_dev = torch.as_tensor([int(t) for t in reference], dtype=torch.int32).to(self.dev)
        force_dev = None
        if force is not None:
            force_dev = torch.where(torch.as_tensor(force["mask"][:n]),
                                    torch.as_tensor(force["tokens"][:n], dtype=torch.int32),
                                    torch.full((n,), -1, dtype=torch.int32)).to(torch.int32).to(self.dev)
        rec = B.struct_tensor(B.ClfOut, n, self.dev)
        sz = C.sizeof(B.ClfOut)
        scratch = B.classify_scratch(self.dev)
        for p in range(n):
            B.disco_draft_step(self.draft, self.kv_d, fed.data_ptr() + 4 * p, 1, self.logits_d, self.ws_d)
            B.disco_classify(self.clf, self.logits_d, self.draft.shape.vocab, float(p + 1), 0.0, 0,
                             rec.data_ptr() + sz * p,
                             force_token=(force_dev.data_ptr() + 4 * p) if force_dev is not None else None,
                             scratch=scratch)
        feats = torch.empty(n, B.N_FEAT, dtype=torch.float32, device=self.dev)
        labels = torch.empty(n, dtype=torch.int32, device=self.dev)
        tokens = torch.empty(n, dtype=torch.int32, device=self.dev)
        B.disco_clf_examples(rec, n, ref_dev, feats, labels, tokens)
        torch.cuda.synchronize(self.dev)
        return feats, labels, tokens


    def generate(self, prompt: Sequence[int], max_new: int, policy: Dict, force: Optional[Dict] = None,
                 trace: bool = False, do_prefill: bool = True, on_iteration=None,
                 max_iterations: Optional[int] = None) -> Dict:
        mode = policy["mode"]
        assert mode in ("static", "disco", "oracle", "heuristic", "ppl")
        pos_mode = policy.get("pos_mode", "absolute")
        cap_policy = {"static": policy.get("gamma"), "disco": policy.get("sl_max"),
                      "oracle": policy.get("sl_max", B.MAX_BLOCK - 1), "heuristic": policy.get("sl_max"),
                      "ppl": policy.get("sl_max")}[mode]
        tau = float(policy.get("tau", 0.0)) if mode == "disco" else -1.0e30
        # the two rule-based baselines the paper compares with: a lookahead that follows the last
        # iteration's outcome (disco_heuristic_next), and a perplexity threshold (decided on the device)
        heur_sl = int(policy.get("start", 5)) if mode == "heuristic" else 0
        clf = None if mode == "ppl" else self.clf
        ppl_threshold = float(policy["threshold"]) if mode == "ppl" else 0.0
        if do_prefill:
            self.reset()
            self.prefill(prompt[:-1])
        ref_dev = None
        if mode == "oracle":
            # the target's greedy text, known in advance: drafting stops at the first token that leaves it
            ref = torch.as_tensor(list(policy["reference"][:max_new]), dtype=torch.int32)
            ref_dev = torch.cat([ref, torch.full((B.MAX_BLOCK,), -1, dtype=torch.int32)]).to(self.dev)
        force_dev = None
        if force is not None:
            ft = torch.where(torch.as_tensor(force["mask"][:max_new]),
                             torch.as_tensor(force["tokens"][:max_new], dtype=torch.int32),
                             torch.full((max_new,), -1, dtype=torch.int32))
            force_dev = torch.cat([ft.to(torch.int32), torch.full((B.MAX_BLOCK,), -1, dtype=torch.int32)]).to(self.dev)
        seq = [int(t) for t in prompt]
        n_prompt = len(seq)
        iters: List[Dict] = []
        n_draft_fwd = n_target_fwd = 0
        bufs = B.iter_buffers(self.tok_in, self.logits_d if self.draft is not None else None, self.steps, self.loop_dev,
                              self.loop_host, self.argmax, self.acc_dev, self.acc_host)
        res = B.IterResult()
        chunk = int(policy.get("chunk", 0))
        kv_d, ws_d = (self.kv_d, self.ws_d) if self.draft is not None else (None, None)
        while len(seq) - n_prompt < max_new:
            if max_iterations is not None and len(iters) >= max_iterations:
                break
            emitted = len(seq) - n_prompt
            remaining = max_new - emitted
            cap = min(cap_policy, remaining - 1) if self.draft is not None else 0
            if mode == "heuristic":
                cap = min(cap, heur_sl)
            cap = max(cap, 0)
            ctx_t = self.kv_t.len
            pending = seq[self.kv_d.len:] if cap >= 1 else seq[-1:]
            assert 1 <= len(pending) <= 2
            # the whole iteration (chunks of draft steps, verification, acceptance, both rollbacks) runs in the library
            B.disco_iterate(self.target, self.kv_t, self.ws_t, self.draft, kv_d, ws_d, clf, pending, cap,
                            cap if mode in ("static", "heuristic") else 0, chunk,
                            float(emitted + 1) if pos_mode == "absolute" else 1.0, tau, bufs, res,
                            force_tokens=(force_dev.data_ptr() + 4 * emitted) if force_dev is not None else None,
                            ref_tokens=(ref_dev.data_ptr() + 4 * emitted) if ref_dev is not None else None,
                            ppl_threshold=ppl_threshold)
            sl, n = res.sl, res.n
            block = list(res.block[:sl + 1])
            n_draft_fwd += res.draft_forwards
            n_target_fwd += 1
            steps_rec = None
            if trace and cap >= 1:
                raw = self.steps.cpu().numpy().tobytes()
                sz = C.sizeof(B.ClfOut)
                steps_rec = [B.ClfOut.from_buffer_copy(raw[i * sz:(i + 1) * sz]) for i in range(res.draft_forwards)]
            emit = list(res.emit[:n + 1])[:remaining]
            seq.extend(emit)
            if mode == "heuristic":
                heur_sl = B.disco_heuristic_next(heur_sl, sl, n, int(policy.get("up", 2)), int(policy.get("down", 1)), cap_policy)
            it = {"sl": sl, "n": n, "block": block, "emit": emit, "ctx": ctx_t}
            if trace:
                it["target_argmax"] = self.argmax[:sl + 1].tolist()
                it["steps"] = steps_rec
            iters.append(it)
            if on_iteration is not None:
                on_iteration(it)
        hist: Dict[int, int] = {}
        for it in iters:
            hist[it["sl"]] = hist.get(it["sl"], 0) + 1
        return {"tokens": seq[n_prompt:], "iterations": iters, "n_iterations": len(iters),
                "n_draft_forwards": n_draft_fwd, "n_target_forwards": n_target_fwd,
                "sl_hist": dict(sorted(hist.items()))}

    def generate_sampling(self, prompt: Sequence[int], max_new: int, policy: Dict, temperature: float,
                          uniforms: Dict, do_prefill: bool = True, on_iteration=None,
                          max_iterations: Optional[int] = None) -> Dict:
        """The loop at temperature > 0: sampled draft tokens, speculative-sampling acceptance.
        uniforms: {"draft", "accept", "resample"}: float32 tensors indexed by generated position (at
        least max_new + cap entries); they are copied to the device once."""
        mode = policy["mode"]
        assert mode in ("static", "disco")
        pos_mode = policy.get("pos_mode", "absolute")
        cap_policy = policy["gamma"] if mode == "static" else policy["sl_max"]
        tau = float(policy.get("tau", 0.0))
        vocab = self.target.shape.vocab
        if do_prefill:
            self.reset()
            self.prefill(prompt[:-1])
        pad = torch.zeros(B.MAX_BLOCK, dtype=torch.float32)
        u_dev = {k: torch.cat([uniforms[k].to(torch.float32), pad]).to(self.dev) for k in ("draft", "accept", "resample")}
        q_rows = torch.zeros(B.MAX_BLOCK, vocab, dtype=torch.float32, device=self.dev)
        t_logits = torch.zeros(B.MAX_BLOCK, vocab, dtype=torch.float32, device=self.dev)
        seq = [int(t) for t in prompt]
        n_prompt = len(seq)
        iters: List[Dict] = []
        loop_block_ptr = self.loop_dev.data_ptr() + 4
        while len(seq) - n_prompt < max_new:
            if max_iterations is not None and len(iters) >= max_iterations:
                break
            emitted = len(seq) - n_prompt
            remaining = max_new - emitted
            cap = min(cap_policy, remaining - 1)
            ctx_t = self.kv_t.len
            if cap >= 1:
                len_d0 = self.kv_d.len
                pending = seq[len_d0:]
                assert 1 <= len(pending) <= 2
                self._put_tokens(pending)
                B.disco_draft_loop_sampled(self.draft, self.kv_d, self.clf, self.tok_in, len(pending), cap,
                                           cap if mode == "static" else 0,
                                           float(emitted + 1) if pos_mode == "absolute" else 1.0, tau, temperature,
                                           u_dev["draft"].data_ptr() + 4 * emitted, q_rows, self.logits_d,
                                           self.steps, self.loop_dev, self.loop_host, self.ws_d)
                torch.cuda.current_stream().synchronize()
                lo = B.LoopOut.from_buffer_copy(self.loop_host.numpy().tobytes())
                sl = lo.sl
                block = list(lo.block[:sl + 1])
                B.disco_kv_rollback(self.kv_d, len_d0 + len(pending) + sl - 1)
            else:
                sl, block = 0, [seq[-1]]
                lo = B.LoopOut()
                lo.sl = 0
                lo.block[0] = seq[-1]
                self.loop_dev.copy_(torch.frombuffer(bytearray(bytes(lo)), dtype=torch.uint8))
            B.disco_verify(self.target, self.kv_t, loop_block_ptr, sl + 1, self.argmax, t_logits, self.ws_t)
            B.disco_accept_sample(loop_block_ptr, sl + 1, q_rows, t_logits, vocab, temperature,
                                  u_dev["accept"].data_ptr() + 4 * emitted, u_dev["resample"].data_ptr() + 4 * emitted,
                                  self.acc_dev, self.acc_host)
            torch.cuda.current_stream().synchronize()
            acc = B.AcceptOut.from_buffer_copy(self.acc_host.numpy().tobytes())
            n = acc.n
            emit = list(acc.emit[:n + 1])[:remaining]
            seq.extend(emit)
            B.disco_kv_rollback(self.kv_t, ctx_t + n + 1)
            if self.draft is not None and self.kv_d.len > ctx_t + n + 1:
                B.disco_kv_rollback(self.kv_d, ctx_t + n + 1)
            iters.append({"sl": sl, "n": n, "block": block, "emit": emit, "ctx": ctx_t})
            if on_iteration is not None:
                on_iteration(iters[-1])
        hist: Dict[int, int] = {}
        for it in iters:
            hist[it["sl"]] = hist.get(it["sl"], 0) + 1
        return {"tokens": seq[n_prompt:], "iterations": iters, "n_iterations": len(iters),
                "sl_hist": dict(sorted(hist.items()))}
