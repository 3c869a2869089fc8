"""Selective-rollout decode for MI355X: thin ctypes binding over libsr.so (see include/sr.h).

Argument marshalling only -- every step of the path runs in the library's HIP kernels.  PyTorch
is used by callers for device memory and streams; this module never computes anything itself and
there is no CPU fallback: if libsr.so is missing and cannot be built, loading fails.
"""
from __future__ import annotations

import ctypes
import os

from .build import LIB, build

_lib = None

SR_OK, SR_E_ARG, SR_E_NOMEM, SR_E_STATE, SR_E_HIP, SR_E_LIMIT = 0, -1, -2, -3, -4, -5
GRPO_STATIC_MAX_GROUPS = 65536

EXPORTS = ("sr_init", "sr_destroy", "sr_load_weights", "sr_prefill_chunk", "sr_decode_step", "sr_gate",
           "sr_retire_and_compact", "sr_gate_batch", "sr_set_actions", "sr_get_actions", "sr_get_logits",
           "sr_get_live_map", "sr_stats", "sr_strerror", "sr_profile", "sr_profile_read", "sr_signals_batch",
           "sr_score_chunk", "sr_get_logprob", "sr_grpo_loss", "sr_finish_sequences", "sr_grpo_loss_static",
           "sr_probe_hbm", "sr_probe_mfma_bf16", "sr_probe_mfma_under_loads", "sr_gate_batch_antidiag",
           "sr_probe_decode_attention")

KERNEL_CLASSES = ("norm", "gemm_qkv", "qkv_post", "attn_decode", "attn_prefill", "attn_merge",
                  "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm_head", "argmax")


class SrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


class ModelShape(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("hidden", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("ffn", ctypes.c_int32),
                ("vocab", ctypes.c_int32), ("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float),
                ("qkv_bias", ctypes.c_int32), ("tied_lm_head", ctypes.c_int32)]


class Options(ctypes.Structure):
    _fields_ = [("page_tokens", ctypes.c_int32), ("max_seq_len", ctypes.c_int32), ("max_turns", ctypes.c_int32),
                ("action_mod", ctypes.c_int32), ("max_prefill_rows", ctypes.c_int32),
                ("kv_pool_bytes", ctypes.c_uint64), ("temperature", ctypes.c_float),
                ("sample_seed", ctypes.c_uint64), ("tau_H", ctypes.c_float), ("fp32_debug", ctypes.c_int32)]


class LayerWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "bq", "bk", "bv", "norm1", "norm2")]


class Weights(ctypes.Structure):
    _fields_ = [("embed", ctypes.c_void_p), ("lm_head", ctypes.c_void_p), ("final_norm", ctypes.c_void_p),
                ("layers", ctypes.POINTER(LayerWeights))]


class KernelTime(ctypes.Structure):
    _fields_ = [("launches", ctypes.c_int64), ("total_ms", ctypes.c_double)]


class Stats(ctypes.Structure):
    _fields_ = [("decoded_tokens", ctypes.c_int64), ("prefill_tokens", ctypes.c_int64)] + \
               [(n, ctypes.c_int32) for n in ("n_live_groups", "n_live_seq", "seq_len", "turn", "pages_total",
                                              "pages_in_use", "groups_retired", "pages_freed", "cow_page_copies",
                                              "seqs_finished", "groups_finished")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


def lib():
    """Load libsr.so (building it first only if it does not exist)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        L = ctypes.CDLL(LIB)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        L.sr_init.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(ModelShape), ci, ci, ctypes.c_double,
                              ctypes.POINTER(Options)]
        L.sr_destroy.argtypes = [vp]
        L.sr_destroy.restype = None
        L.sr_load_weights.argtypes = [vp, ctypes.POINTER(Weights), vp]
        L.sr_prefill_chunk.argtypes = [vp, vp, ci, ci, vp]
        L.sr_decode_step.argtypes = [vp, vp, vp, vp]
        L.sr_gate.argtypes = [vp, ci, vp, vp, vp]
        L.sr_retire_and_compact.argtypes = [vp, ctypes.POINTER(ci), vp]
        L.sr_gate_batch.argtypes = [vp, ci, ci, ci, ctypes.POINTER(ci), ci, ctypes.c_double, vp, vp, vp]
        L.sr_gate_batch_antidiag.argtypes = L.sr_gate_batch.argtypes
        L.sr_signals_batch.argtypes = [vp, vp, vp, ci, ci, ci, ctypes.POINTER(ci), ci, ctypes.c_double,
                                       ctypes.c_double, vp, vp]
        L.sr_score_chunk.argtypes = [vp, vp, vp, ci, vp, vp]
        L.sr_get_logprob.argtypes = [vp, vp, vp]
        L.sr_grpo_loss.argtypes = [vp, vp, ci, ci, ctypes.c_double, vp, vp, vp, vp]
        L.sr_grpo_loss_static.argtypes = [vp, vp, ci, ci, ctypes.c_double, vp, vp, vp]
        L.sr_probe_hbm.argtypes = [vp, vp, ctypes.c_size_t, ci, ci, vp, ctypes.POINTER(ctypes.c_double)]
        L.sr_probe_decode_attention.argtypes = [ci] * 8 + [vp, ctypes.POINTER(ctypes.c_double),
                                                  ctypes.POINTER(ctypes.c_double)]
        L.sr_probe_mfma_bf16.argtypes = [vp, ctypes.c_size_t, ci, vp, ctypes.POINTER(ctypes.c_double)]
        L.sr_probe_mfma_under_loads.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t, ci, ci, ci, ci, vp,
                                                ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.sr_finish_sequences.argtypes = [vp, vp, ctypes.POINTER(ci), vp]
        L.sr_set_actions.argtypes = [vp, ci, vp, vp]
        L.sr_get_actions.argtypes = [vp, vp, vp]
        L.sr_get_logits.argtypes = [vp, vp, vp]
        L.sr_get_live_map.argtypes = [vp, vp]
        L.sr_stats.argtypes = [vp, ctypes.POINTER(Stats)]
        L.sr_profile.argtypes = [vp, ci]
        L.sr_profile_read.argtypes = [vp, ctypes.POINTER(KernelTime), vp]
        L.sr_strerror.argtypes = [ci]
        L.sr_strerror.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("sr_destroy", "sr_strerror"):
                getattr(L, name).restype = ci
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().sr_strerror(status).decode()


def _check(status: int, where: str):
    if status != SR_OK:
        raise SrError(status, where)


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / None."""
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def sr_gate_batch(actions, prefix_lens, threshold: float, sums=None, retire=None, stream=None):
    """actions: device int32 [n_groups, G, stride]; sums int32 / retire uint8: device [n_lens, n_groups]."""
    n_groups, G, stride = actions.shape
    lens = (ctypes.c_int * len(prefix_lens))(*prefix_lens)
    _check(lib().sr_gate_batch(_ptr(actions), n_groups, G, stride, lens, len(prefix_lens), threshold,
                               _ptr(sums), _ptr(retire), _stream(stream)), "sr_gate_batch")


def sr_gate_batch_antidiag(actions, prefix_lens, threshold: float, sums=None, retire=None, stream=None):
    """sr_gate_batch by the anti-diagonal decomposition (same arguments, same results)."""
    n_groups, G, stride = actions.shape
    lens = (ctypes.c_int * len(prefix_lens))(*prefix_lens)
    _check(lib().sr_gate_batch_antidiag(_ptr(actions), n_groups, G, stride, lens, len(prefix_lens), threshold,
                                        _ptr(sums), _ptr(retire), _stream(stream)), "sr_gate_batch_antidiag")


SIGNALS_BYTES = 64       # sizeof(sr_signals_t)
SIGNALS_FIELDS = (("d_K", "f8"), ("lev_scaled", "i8"), ("bigram_jaccard", "f8"), ("action_entropy", "f8"),
                  ("unique_prefix", "i4"), ("n_at_step", "i4"), ("unique_action", "i4"), ("unique_obs", "i4"),
                  ("n_done", "i4"), ("lev_sum", "i4"), ("cut_d", "u1"), ("cut_or", "u1"), ("reserved", "u1", (6,)))


def sr_signals_batch(actions, prefix_lens, d_L: float, tau_H: float, out, obs=None, end_step=None, stream=None):
    """actions, obs: device int32 [n_groups, G, stride]; end_step: device int32 [n_groups, G];
    out: device uint8 [n_lens, n_groups, SIGNALS_BYTES] receiving sr_signals_t records."""
    n_groups, G, stride = actions.shape
    lens = (ctypes.c_int * len(prefix_lens))(*prefix_lens)
    _check(lib().sr_signals_batch(_ptr(actions), _ptr(obs), _ptr(end_step), n_groups, G, stride, lens,
                                  len(prefix_lens), d_L, tau_H, _ptr(out), _stream(stream)), "sr_signals_batch")


def sr_grpo_loss(logprob, rewards, G: int, eps: float, advantages, group_scratch, loss, stream=None):
    """logprob: device float64 [n_groups*G]; rewards: device float32, same; advantages: device float32 or None;
    group_scratch: device float64 [n_groups]; loss: device float64 [1]."""
    n_groups = logprob.numel() // G
    _check(lib().sr_grpo_loss(_ptr(logprob), _ptr(rewards), n_groups, G, eps, _ptr(advantages), _ptr(group_scratch),
                              _ptr(loss), _stream(stream)), "sr_grpo_loss")


def sr_grpo_loss_static(logprob, rewards, G: int, eps: float, advantages, loss, stream=None):
    """sr_grpo_loss without a workspace argument (the library's fixed device array holds the group shares)."""
    n_groups = logprob.numel() // G
    _check(lib().sr_grpo_loss_static(_ptr(logprob), _ptr(rewards), n_groups, G, eps, _ptr(advantages), _ptr(loss),
                                     _stream(stream)), "sr_grpo_loss_static")


def sr_probe_hbm(src, dst, mode: int, iters: int = 10, stream=None) -> float:
    """GB/s of a streaming read of `src` (mode 0: non-temporal loads, 1: default loads) or of a copy to dst (2)."""
    out = ctypes.c_double()
    nbytes = src.numel() * src.element_size()
    _check(lib().sr_probe_hbm(_ptr(src), _ptr(dst), nbytes, mode, iters, _stream(stream), ctypes.byref(out)),
           "sr_probe_hbm")
    return out.value


def sr_probe_decode_attention(n_groups: int, G: int, shared_tokens: int, priv_tokens: int, priv_splits: int,
                              phases: int, hot: bool = False, iters: int = 24, stream=None):
    """(microseconds per launch, K/V bytes per launch) of one layer's decode attention on synthetic pages;
    phases: 1 shared prompt, 2 private, 3 both in one launch, +4 with the merge launch behind it."""
    us, nbytes = ctypes.c_double(), ctypes.c_double()
    _check(lib().sr_probe_decode_attention(n_groups, G, shared_tokens, priv_tokens, priv_splits, phases, int(hot), iters,
                                           _stream(stream), ctypes.byref(us), ctypes.byref(nbytes)),
           "sr_probe_decode_attention")
    return us.value, nbytes.value


def sr_probe_mfma_bf16(scratch, iters: int = 3, stream=None) -> float:
    """TFLOP/s of a register-resident bf16 matrix-core loop."""
    out = ctypes.c_double()
    _check(lib().sr_probe_mfma_bf16(_ptr(scratch), scratch.numel() * scratch.element_size(), iters, _stream(stream),
                                    ctypes.byref(out)), "sr_probe_mfma_bf16")
    return out.value


def sr_probe_mfma_under_loads(buf, scratch, path: int, loads_per_16: int, lds_reads: bool = False, iters: int = 3,
                              stream=None):
    """(TFLOP/s of the matrix loop, GB/s of the loads beside it); path 0 none, 1 into registers, 2 straight into LDS."""
    tf, gb = ctypes.c_double(), ctypes.c_double()
    _check(lib().sr_probe_mfma_under_loads(_ptr(buf), buf.numel() * buf.element_size(), _ptr(scratch),
                                           scratch.numel() * scratch.element_size(), path, loads_per_16, int(lds_reads),
                                           iters, _stream(stream), ctypes.byref(tf), ctypes.byref(gb)),
           "sr_probe_mfma_under_loads")
    return tf.value, gb.value


class Context:
    """Owns one sr_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, shape, n_groups: int, G: int, threshold: float, *, page_tokens=64, max_seq_len=4096,
                 max_turns=32, action_mod=64, max_prefill_rows=0, kv_pool_bytes=1 << 30, temperature=0.0,
                 sample_seed=0, tau_H=0.0, fp32_debug=False, tied_lm_head=False):
        self.shape = ModelShape(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                                shape.ffn, shape.vocab, shape.rms_eps, shape.rope_theta, int(shape.qkv_bias),
                                int(tied_lm_head))
        self.opt = Options(page_tokens, max_seq_len, max_turns, action_mod, max_prefill_rows, kv_pool_bytes,
                           temperature, sample_seed, tau_H, int(fp32_debug))
        self.G, self.n_groups0, self.vocab, self.max_turns = G, n_groups, shape.vocab, max_turns
        self._h = ctypes.c_void_p()
        _check(lib().sr_init(ctypes.byref(self._h), ctypes.byref(self.shape), n_groups, G, threshold,
                             ctypes.byref(self.opt)), "sr_init")

    def close(self):
        if self._h:
            lib().sr_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def sr_load_weights(self, embed, lm_head, final_norm, layers, stream=None):
        """layers: list of dicts name -> device bf16 tensor (names as in sr_layer_weights)."""
        arr = (LayerWeights * len(layers))()
        for i, d in enumerate(layers):
            for name, _ in LayerWeights._fields_:
                setattr(arr[i], name, _ptr(d.get(name)))
        w = Weights(_ptr(embed), _ptr(lm_head), _ptr(final_norm), arr)
        _check(lib().sr_load_weights(self._h, ctypes.byref(w), _stream(stream)), "sr_load_weights")

    def sr_prefill_chunk(self, tokens, shared_per_group: bool, stream=None):
        _check(lib().sr_prefill_chunk(self._h, _ptr(tokens), tokens.shape[-1], int(shared_per_group),
                                      _stream(stream)), "sr_prefill_chunk")

    def sr_score_chunk(self, tokens, action_mask=None, out_token_logprob=None, stream=None):
        _check(lib().sr_score_chunk(self._h, _ptr(tokens), _ptr(action_mask), tokens.shape[-1],
                                    _ptr(out_token_logprob), _stream(stream)), "sr_score_chunk")

    def sr_get_logprob(self, dst, stream=None):
        _check(lib().sr_get_logprob(self._h, _ptr(dst), _stream(stream)), "sr_get_logprob")

    def sr_decode_step(self, forced=None, out_tokens=None, stream=None):
        _check(lib().sr_decode_step(self._h, _ptr(forced), _ptr(out_tokens), _stream(stream)), "sr_decode_step")

    def sr_gate(self, turn: int, out_sums=None, out_retire=None, stream=None):
        _check(lib().sr_gate(self._h, turn, _ptr(out_sums), _ptr(out_retire), _stream(stream)), "sr_gate")

    def sr_finish_sequences(self, host_done, stream=None) -> int:
        """host_done: numpy uint8 [n_live_seq]; returns the number of sequences left."""
        import numpy as np
        d = np.ascontiguousarray(host_done, dtype=np.uint8)
        n = ctypes.c_int(-1)
        _check(lib().sr_finish_sequences(self._h, d.ctypes.data, ctypes.byref(n), _stream(stream)),
               "sr_finish_sequences")
        return n.value

    def sr_retire_and_compact(self, stream=None) -> int:
        n = ctypes.c_int(-1)
        _check(lib().sr_retire_and_compact(self._h, ctypes.byref(n), _stream(stream)), "sr_retire_and_compact")
        return n.value

    def sr_set_actions(self, turn: int, ids, stream=None):
        _check(lib().sr_set_actions(self._h, turn, _ptr(ids), _stream(stream)), "sr_set_actions")

    def sr_get_actions(self, dst, stream=None):
        _check(lib().sr_get_actions(self._h, _ptr(dst), _stream(stream)), "sr_get_actions")

    def sr_get_logits(self, dst, stream=None):
        _check(lib().sr_get_logits(self._h, _ptr(dst), _stream(stream)), "sr_get_logits")

    def sr_get_live_map(self):
        import numpy as np
        n = self.sr_stats()["n_live_seq"]
        out = np.zeros(max(n, 1), dtype=np.int32)
        _check(lib().sr_get_live_map(self._h, out.ctypes.data), "sr_get_live_map")
        return out[:n]

    def sr_profile(self, enable: bool):
        _check(lib().sr_profile(self._h, int(enable)), "sr_profile")

    def sr_profile_read(self, stream=None) -> dict:
        arr = (KernelTime * len(KERNEL_CLASSES))()
        _check(lib().sr_profile_read(self._h, arr, _stream(stream)), "sr_profile_read")
        return {KERNEL_CLASSES[i]: (arr[i].launches, arr[i].total_ms) for i in range(len(KERNEL_CLASSES))}

    def sr_stats(self) -> dict:
        s = Stats()
        _check(lib().sr_stats(self._h, ctypes.byref(s)), "sr_stats")
        return s.as_dict()
