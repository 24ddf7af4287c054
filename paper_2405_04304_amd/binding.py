"""ctypes binding of include/disco.h: the same entry points under the same names, plus small
holders that keep the PyTorch-allocated device buffers of a model, a KV cache and a workspace alive.
No arithmetic of the method happens here."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdisco.so")

MAX_BLOCK = 16
N_FEAT = 12
FAMILY = {"A": 0, "B": 1}
OK, EINVAL, ECAP, ESTATE, EHIP = 0, -1, -2, -3, -4


class DiscoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"disco error {code}: {msg}")
        self.code = code


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("family", "n_layers", "d_model", "n_heads", "d_head",
                                         "n_kv_heads", "d_ff", "vocab", "max_pos")] + \
               [("norm_eps", C.c_float), ("rope_base", C.c_float)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("norm1_g", "norm1_b", "wqkv", "wo", "norm2_g", "norm2_b",
                                          "w_in", "w_out")]


class ModelWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("tok_emb_stride", C.c_int64), ("pos_emb", C.c_void_p),
                ("layers", C.POINTER(LayerWeights)), ("normf_g", C.c_void_p), ("normf_b", C.c_void_p),
                ("wlm", C.c_void_p)]


class Clf(C.Structure):
    _fields_ = [("dev_params", C.c_void_p), ("hidden", C.c_int32)]


class ClfOut(C.Structure):
    _fields_ = [("token", C.c_int32), ("feats", C.c_float * N_FEAT), ("score", C.c_float),
                ("halt", C.c_uint32), ("executed", C.c_uint32)]


class AcceptOut(C.Structure):
    _fields_ = [("n", C.c_int32), ("n_emit", C.c_int32), ("emit", C.c_int32 * MAX_BLOCK)]


class LoopOpts(C.Structure):
    _fields_ = [("dev_force_tokens", C.c_void_p), ("dev_ref_tokens", C.c_void_p), ("temperature", C.c_float),
                ("dev_u_draft", C.c_void_p), ("dev_draft_probs", C.c_void_p), ("ppl_threshold", C.c_float),
                ("block_offset", C.c_int32), ("open_end", C.c_int32)]


class LoopOut(C.Structure):
    _fields_ = [("sl", C.c_int32), ("block", C.c_int32 * MAX_BLOCK), ("halted", C.c_int32)]


class IterBuffers(C.Structure):
    _fields_ = [("dev_tokens_in", C.c_void_p), ("dev_logits_draft", C.c_void_p), ("dev_steps", C.c_void_p),
                ("dev_loop_out", C.c_void_p), ("host_loop_out", C.c_void_p), ("dev_argmax", C.c_void_p),
                ("dev_accept_out", C.c_void_p), ("host_accept_out", C.c_void_p)]


class IterResult(C.Structure):
    _fields_ = [("sl", C.c_int32), ("n", C.c_int32), ("draft_forwards", C.c_int32),
                ("draft_steps_enqueued", C.c_int32), ("block", C.c_int32 * MAX_BLOCK), ("emit", C.c_int32 * MAX_BLOCK)]


_SIGNATURES = {
    "disco_last_error": (C.c_char_p, []),
    "disco_pack_weight": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "disco_pack_gate_up": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "disco_model_create": (C.c_int, [C.POINTER(ModelDesc), C.POINTER(ModelWeights), C.POINTER(C.c_void_p)]),
    "disco_model_destroy": (None, [C.c_void_p]),
    "disco_kv_bytes": (C.c_size_t, [C.c_void_p, C.c_int, C.c_int]),
    "disco_kv_create": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_int,
                                  C.POINTER(C.c_int32), C.POINTER(C.c_void_p)]),
    "disco_kv_destroy": (None, [C.c_void_p]),
    "disco_kv_len": (C.c_int, [C.c_void_p]),
    "disco_kv_pages_in_use": (C.c_int, [C.c_void_p]),
    "disco_kv_fill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]),
    "disco_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int, C.c_int]),
    "disco_workspace_init": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_void_p]),
    "disco_prefill_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int, C.c_int]),
    "disco_prefill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t,
                                C.c_void_p]),
    "disco_prefill_ex": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_uint, C.c_void_p,
                                   C.c_size_t, C.c_void_p]),
    "disco_draft_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                                   C.c_size_t, C.c_void_p, C.c_void_p]),
    "disco_classify": (C.c_int, [C.POINTER(Clf), C.c_void_p, C.c_int, C.c_float, C.c_float, C.c_int,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_void_p]),
    "disco_classify_scratch_init": (C.c_int, [C.c_void_p, C.c_void_p]),
    "disco_classify_static": (C.c_int, [C.POINTER(Clf), C.c_void_p, C.c_int, C.c_float, C.c_float, C.c_int,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p]),
    "disco_verify": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                               C.c_void_p, C.c_size_t, C.c_void_p]),
    "disco_accept": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                               C.c_void_p]),
    "disco_kv_rollback": (C.c_int, [C.c_void_p, C.c_int]),
    "disco_draft_loop": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(Clf), C.c_void_p, C.c_int, C.c_int,
                                   C.c_int, C.c_float, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "disco_sample": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_float, C.c_void_p, C.c_void_p,
                               C.c_void_p, C.c_void_p]),
    "disco_accept_sample": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                      C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "disco_draft_loop_sampled": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(Clf), C.c_void_p, C.c_int, C.c_int,
                                           C.c_int, C.c_float, C.c_float, C.c_float, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_size_t, C.c_void_p]),
    "disco_draft_loop_ex": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(Clf), C.c_void_p, C.c_int, C.c_int,
                                      C.c_int, C.c_float, C.c_float, C.POINTER(LoopOpts), C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "disco_iterate": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_size_t, C.POINTER(Clf), C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_int, C.c_int,
                                C.c_float, C.c_float, C.POINTER(LoopOpts), C.POINTER(IterBuffers),
                                C.POINTER(IterResult), C.c_void_p]),
    "disco_clf_train": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float, C.c_void_p,
                                  C.c_void_p, C.c_void_p]),
    "disco_clf_eval": (C.c_int, [C.POINTER(Clf), C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_void_p,
                                 C.c_void_p, C.c_void_p]),
    "disco_set_launch_mode": (C.c_int, [C.c_int]),
    "disco_clf_examples": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "disco_heuristic_next": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "disco_probe_enable": (C.c_int, [C.c_int]),
    "disco_probe_read_ms": (C.c_float, []),
    "disco_set_wait_limit": (C.c_int, [C.c_int]),
}
EXPORTS = sorted(_SIGNATURES)

_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Fails loudly when it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2405_04304_amd.build` "
                               "(there is no CPU or PyTorch fallback for the DISCO kernels)")
        _lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(_lib, name)
            fn.restype, fn.argtypes = res, args
    return _lib


def last_error() -> str:
    return lib().disco_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise DiscoError(rc, last_error())


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


# ---- the C entry points, same names, tensors or raw addresses accepted -----------------------

def disco_pack_weight(src, n, k, dst, stream=None):
    _check(lib().disco_pack_weight(_ptr(src), n, k, _ptr(dst), _stream() if stream is None else stream))


def disco_pack_gate_up(gate, up, d_ff, k, dst, stream=None):
    _check(lib().disco_pack_gate_up(_ptr(gate), _ptr(up), d_ff, k, _ptr(dst),
                                    _stream() if stream is None else stream))


def disco_draft_step(model, kv, tokens_in, n_in, logits, ws, gate=None, stream=None):
    _check(lib().disco_draft_step(model.handle, kv.handle, _ptr(tokens_in), n_in, _ptr(logits),
                                  _ptr(ws.buf), ws.nbytes, _ptr(gate),
                                  _stream() if stream is None else stream))


def disco_classify(clf, logits, vocab, pos_feature, tau, force_halt, out, token_next=None,
                   block_slot=None, gate=None, sl_count=None, force_token=None, scratch=None, stream=None):
    _check(lib().disco_classify(C.byref(clf.c) if clf is not None else None, _ptr(logits), vocab,
                                pos_feature, tau, int(force_halt), _ptr(out), _ptr(token_next),
                                _ptr(block_slot), _ptr(gate), _ptr(sl_count), _ptr(force_token), _ptr(scratch),
                                _stream() if stream is None else stream))


def disco_classify_static(clf, logits, vocab, pos_feature, tau, force_halt, out, token_next=None,
                          block_slot=None, gate=None, sl_count=None, force_token=None, stream=None):
    _check(lib().disco_classify_static(C.byref(clf.c) if clf is not None else None, _ptr(logits), vocab,
                                       pos_feature, tau, int(force_halt), _ptr(out), _ptr(token_next),
                                       _ptr(block_slot), _ptr(gate), _ptr(sl_count), _ptr(force_token),
                                       _stream() if stream is None else stream))


CLASSIFY_SCRATCH_BYTES = 4352


def classify_scratch(device="cuda") -> torch.Tensor:
    """Device scratch for the many-workgroup form of disco_classify, ticket word zeroed."""
    t = torch.empty(CLASSIFY_SCRATCH_BYTES, dtype=torch.uint8, device=device)
    _check(lib().disco_classify_scratch_init(t.data_ptr(), _stream()))
    return t


def disco_verify(model, kv, block, n_block, argmax, logits, ws, stream=None):
    _check(lib().disco_verify(model.handle, kv.handle, _ptr(block), n_block, _ptr(argmax), _ptr(logits),
                              _ptr(ws.buf), ws.nbytes, _stream() if stream is None else stream))


PREFILL_BF16_ACTIVATIONS = 1


def disco_prefill(model, kv, tokens, n_tokens, logits_last, ws, stream=None, flags=0):
    if flags:
        _check(lib().disco_prefill_ex(model.handle, kv.handle, _ptr(tokens), n_tokens, _ptr(logits_last), flags,
                                      _ptr(ws.buf), ws.nbytes, _stream() if stream is None else stream))
        return
    _check(lib().disco_prefill(model.handle, kv.handle, _ptr(tokens), n_tokens, _ptr(logits_last), _ptr(ws.buf),
                               ws.nbytes, _stream() if stream is None else stream))


def disco_accept(block, argmax, n_block, out, host_out=None, dev_n_block=None, stream=None):
    _check(lib().disco_accept(_ptr(block), _ptr(argmax), n_block, _ptr(dev_n_block), _ptr(out),
                              _ptr(host_out), _stream() if stream is None else stream))


def disco_kv_rollback(kv, new_len):
    _check(lib().disco_kv_rollback(kv.handle, new_len))


def disco_draft_loop(model, kv, clf, tokens_in, n_in, cap, static_sl, pos_feature0, tau, force_tokens,
                     logits, steps, out, host_out, ws, stream=None):
    _check(lib().disco_draft_loop(model.handle, kv.handle, C.byref(clf.c) if clf is not None else None,
                                  _ptr(tokens_in), n_in, cap, static_sl, pos_feature0, tau,
                                  _ptr(force_tokens), _ptr(logits), _ptr(steps), _ptr(out),
                                  _ptr(host_out), _ptr(ws.buf), ws.nbytes,
                                  _stream() if stream is None else stream))


def disco_draft_loop_ex(model, kv, clf, tokens_in, n_in, cap, static_sl, pos_feature0, tau, logits, steps, out,
                        host_out, ws, force_tokens=None, ref_tokens=None, temperature=0.0, u_draft=None,
                        draft_probs=None, ppl_threshold=0.0, block_offset=0, open_end=0, stream=None):
    opts = LoopOpts(_ptr(force_tokens), _ptr(ref_tokens), temperature, _ptr(u_draft), _ptr(draft_probs),
                    ppl_threshold, block_offset, open_end)
    _check(lib().disco_draft_loop_ex(model.handle, kv.handle, C.byref(clf.c) if clf is not None else None,
                                     _ptr(tokens_in), n_in, cap, static_sl, pos_feature0, tau, C.byref(opts),
                                     _ptr(logits), _ptr(steps), _ptr(out), _ptr(host_out), _ptr(ws.buf), ws.nbytes,
                                     _stream() if stream is None else stream))


def iter_buffers(tokens_in, logits_draft, steps, loop_out, host_loop_out, argmax, accept_out, host_accept_out):
    return IterBuffers(_ptr(tokens_in), _ptr(logits_draft), _ptr(steps), _ptr(loop_out), _ptr(host_loop_out),
                       _ptr(argmax), _ptr(accept_out), _ptr(host_accept_out))


def disco_iterate(target, kv_t, ws_t, draft, kv_d, ws_d, clf, pending, cap, static_sl, chunk, pos_feature0, tau,
                  buffers, result, force_tokens=None, ref_tokens=None, ppl_threshold=0.0, stream=None):
    """One speculative iteration in the library; `result` (IterResult) is filled on return."""
    opts = LoopOpts(_ptr(force_tokens), _ptr(ref_tokens), 0.0, None, None, ppl_threshold, 0, 0)
    pend = (C.c_int32 * len(pending))(*pending)
    _check(lib().disco_iterate(target.handle, kv_t.handle, _ptr(ws_t.buf), ws_t.nbytes,
                               draft.handle if draft is not None else None, kv_d.handle if kv_d is not None else None,
                               _ptr(ws_d.buf) if ws_d is not None else None, ws_d.nbytes if ws_d is not None else 0,
                               C.byref(clf.c) if clf is not None else None, pend, len(pending), cap, static_sl, chunk,
                               pos_feature0, tau, C.byref(opts), C.byref(buffers), C.byref(result),
                               _stream() if stream is None else stream))


def disco_sample(logits, n_rows, vocab, ld_logits, temperature, u, probs, tokens, stream=None):
    _check(lib().disco_sample(_ptr(logits), n_rows, vocab, ld_logits, temperature, _ptr(u), _ptr(probs),
                              _ptr(tokens), _stream() if stream is None else stream))


def disco_accept_sample(block, n_block, draft_probs, target_logits, vocab, temperature, u_accept, u_resample,
                        out, host_out=None, dev_n_block=None, stream=None):
    _check(lib().disco_accept_sample(_ptr(block), n_block, _ptr(dev_n_block), _ptr(draft_probs),
                                     _ptr(target_logits), vocab, temperature, _ptr(u_accept), _ptr(u_resample),
                                     _ptr(out), _ptr(host_out), _stream() if stream is None else stream))


def disco_draft_loop_sampled(model, kv, clf, tokens_in, n_in, cap, static_sl, pos_feature0, tau, temperature,
                             u_draft, draft_probs, logits, steps, out, host_out, ws, stream=None):
    _check(lib().disco_draft_loop_sampled(model.handle, kv.handle, C.byref(clf.c) if clf is not None else None,
                                          _ptr(tokens_in), n_in, cap, static_sl, pos_feature0, tau, temperature,
                                          _ptr(u_draft), _ptr(draft_probs), _ptr(logits), _ptr(steps), _ptr(out),
                                          _ptr(host_out), _ptr(ws.buf), ws.nbytes,
                                          _stream() if stream is None else stream))


TRAIN_MAX_N = 2560
PREFILL_MAX = 8192


def disco_clf_train(feats, labels, n, hidden, epochs, lr, params, loss=None, stream=None):
    _check(lib().disco_clf_train(_ptr(feats), _ptr(labels), n, hidden, epochs, lr, _ptr(params), _ptr(loss),
                                 _stream() if stream is None else stream))


def disco_clf_eval(clf, feats, labels, n, tau, scores=None, counts=None, stream=None):
    _check(lib().disco_clf_eval(C.byref(clf.c), _ptr(feats), _ptr(labels), n, tau, _ptr(scores), _ptr(counts),
                                _stream() if stream is None else stream))


def disco_clf_examples(records, n, ref_tokens, feats, labels, tokens=None, stream=None):
    _check(lib().disco_clf_examples(_ptr(records), n, _ptr(ref_tokens), _ptr(feats), _ptr(labels), _ptr(tokens),
                                    _stream() if stream is None else stream))


def disco_heuristic_next(lookahead: int, drafted: int, accepted: int, up: int, down: int, cap: int) -> int:
    r = lib().disco_heuristic_next(lookahead, drafted, accepted, up, down, cap)
    if r < 0:
        raise DiscoError(r, last_error())
    return r


def disco_set_launch_mode(mode: int) -> int:
    prev = lib().disco_set_launch_mode(mode)
    if prev < 0:
        raise DiscoError(prev, last_error())
    return prev


def disco_set_wait_limit(polls: int) -> int:
    return int(lib().disco_set_wait_limit(polls))


def disco_probe_enable(layer: int) -> None:
    _check(lib().disco_probe_enable(layer))


def disco_probe_read_ms() -> float:
    return float(lib().disco_probe_read_ms())


# ---- holders of device memory ------------------------------------------------------------------

class DiscoModel:
    """Packs a dict of row-major weights (names as in workloads.weight_specs) on the device and owns
    the packed buffers and the library handle."""

    def __init__(self, shape, weights: Dict[str, torch.Tensor], device="cuda", tok_emb=None,
                 tok_emb_stride: Optional[int] = None):
        self.shape = shape
        self.device = torch.device(device)
        self._keep = []
        fam_a = shape.family == "A"

        def dev(t, dtype):
            t = t.to(self.device, dtype=dtype).contiguous()
            self._keep.append(t)
            return t

        def packed(name):
            src = weights[name].to(self.device, dtype=torch.bfloat16).contiguous()
            dst = torch.empty_like(src)
            disco_pack_weight(src, src.shape[0], src.shape[1], dst)
            self._keep.append(dst)
            return dst

        layers = (LayerWeights * shape.n_layers)()
        for l in range(shape.n_layers):
            p = f"l{l}."
            L = layers[l]
            L.norm1_g = dev(weights[p + "norm1_g"], torch.float32).data_ptr()
            L.norm2_g = dev(weights[p + "norm2_g"], torch.float32).data_ptr()
            if fam_a:
                L.norm1_b = dev(weights[p + "norm1_b"], torch.float32).data_ptr()
                L.norm2_b = dev(weights[p + "norm2_b"], torch.float32).data_ptr()
                L.w_in = packed(p + "w1").data_ptr()
                L.w_out = packed(p + "w2").data_ptr()
            else:
                wg = weights[p + "wg"].to(self.device, dtype=torch.bfloat16).contiguous()
                wu = weights[p + "wu"].to(self.device, dtype=torch.bfloat16).contiguous()
                dst = torch.empty((2 * shape.d_ff, shape.d_model), dtype=torch.bfloat16, device=self.device)
                disco_pack_gate_up(wg, wu, shape.d_ff, shape.d_model, dst)
                self._keep.append(dst)
                L.w_in = dst.data_ptr()
                L.w_out = packed(p + "wd").data_ptr()
            L.wqkv = packed(p + "wqkv").data_ptr()
            L.wo = packed(p + "wo").data_ptr()
        torch.cuda.synchronize(self.device)       # packing sources may now be freed
        self._layers = layers
        mw = ModelWeights()
        emb = tok_emb if tok_emb is not None else dev(weights["tok_emb"], torch.bfloat16)
        self._keep.append(emb)
        self.tok_emb = emb                     # a draft may share this table (see tok_emb / tok_emb_stride)
        mw.tok_emb = emb.data_ptr()
        mw.tok_emb_stride = tok_emb_stride if tok_emb_stride is not None else emb.shape[1]
        mw.pos_emb = dev(weights["pos_emb"], torch.bfloat16).data_ptr() if fam_a else None
        mw.layers = layers
        mw.normf_g = dev(weights["normf_g"], torch.float32).data_ptr()
        mw.normf_b = dev(weights["normf_b"], torch.float32).data_ptr() if fam_a else None
        mw.wlm = packed("wlm").data_ptr()
        torch.cuda.synchronize(self.device)
        desc = ModelDesc(FAMILY[shape.family], shape.n_layers, shape.d_model, shape.n_heads, shape.d_head,
                         shape.n_kv_heads, shape.d_ff, shape.vocab, shape.max_pos,
                         shape.ln_eps if fam_a else shape.rms_eps, shape.rope_base)
        h = C.c_void_p()
        _check(lib().disco_model_create(C.byref(desc), C.byref(mw), C.byref(h)))
        self.handle = h

    def workspace(self, max_block: int, max_ctx: int) -> "Workspace":
        n = lib().disco_workspace_bytes(self.handle, max_block, max_ctx)
        if n == 0:
            raise DiscoError(EINVAL, "bad workspace request")
        ws = Workspace(n, self.device)
        _check(lib().disco_workspace_init(self.handle, ws.buf.data_ptr(), n, max_block, max_ctx, _stream()))
        return ws

    def prefill_workspace(self, n_tokens: int, max_ctx: int) -> "Workspace":
        """Workspace of the dense prompt pass (holds the activations of every prompt token)."""
        n = lib().disco_prefill_workspace_bytes(self.handle, n_tokens, max_ctx)
        if n == 0:
            raise DiscoError(EINVAL, "bad prefill workspace request")
        ws = Workspace(n, self.device)
        _check(lib().disco_workspace_init(self.handle, ws.buf.data_ptr(), n, MAX_BLOCK, max_ctx, _stream()))
        return ws

    def close(self):
        if self.handle:
            lib().disco_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Workspace:
    def __init__(self, nbytes: int, device):
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.nbytes = nbytes


class DiscoKV:
    def __init__(self, model: DiscoModel, capacity: int, page_tokens: int = 16, page_order=None):
        self.model = model
        nbytes = lib().disco_kv_bytes(model.handle, capacity, page_tokens)
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=model.device)
        order = None
        if page_order is not None:
            order = (C.c_int32 * len(page_order))(*[int(p) for p in page_order])
        h = C.c_void_p()
        _check(lib().disco_kv_create(model.handle, self.buf.data_ptr(), nbytes, capacity, page_tokens,
                                     order, C.byref(h)))
        self.handle = h

    @property
    def len(self) -> int:
        return lib().disco_kv_len(self.handle)

    @property
    def pages_in_use(self) -> int:
        return lib().disco_kv_pages_in_use(self.handle)

    def fill(self, kv_tensor: torch.Tensor, stream=None):
        """kv_tensor: bf16 [n_layers, 2, ctx, n_kv_heads, d_head] on the device."""
        assert kv_tensor.dtype == torch.bfloat16 and kv_tensor.is_contiguous()
        _check(lib().disco_kv_fill(self.handle, kv_tensor.data_ptr(), kv_tensor.shape[2],
                                   _stream() if stream is None else stream))
        torch.cuda.synchronize()

    def close(self):
        if self.handle:
            lib().disco_kv_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class DiscoClf:
    """Classifier parameters [W1 | b1 | w2 | b2] as one fp32 device vector."""

    def __init__(self, params: Dict[str, torch.Tensor], device="cuda"):
        flat = torch.cat([params["W1"].reshape(-1), params["b1"].reshape(-1), params["w2"].reshape(-1),
                          params["b2"].reshape(-1)]).to(torch.float32)
        self.dev = flat.to(device).contiguous()
        self.hidden = params["W1"].shape[0]
        self.c = Clf(self.dev.data_ptr(), self.hidden)

    def params(self) -> Dict[str, torch.Tensor]:
        """The parameter vector back as host tensors W1, b1, w2, b2."""
        h, v = self.hidden, self.dev.cpu()
        return {"W1": v[:12 * h].view(h, 12).clone(), "b1": v[12 * h:13 * h].clone(), "w2": v[13 * h:14 * h].clone(),
                "b2": v[14 * h:14 * h + 1].clone()}


def struct_tensor(ctype, n: int = 1, device="cuda", pinned: bool = False) -> torch.Tensor:
    """uint8 buffer for n records of a ctypes struct (device, or pinned host)."""
    nbytes = C.sizeof(ctype) * n
    if pinned:
        return torch.zeros(nbytes, dtype=torch.uint8, pin_memory=True)
    return torch.zeros(nbytes, dtype=torch.uint8, device=device)


def read_struct(ctype, t: torch.Tensor, index: int = 0):
    raw = bytes(t.cpu().numpy().tobytes())
    sz = C.sizeof(ctype)
    return ctype.from_buffer_copy(raw[index * sz:(index + 1) * sz])
