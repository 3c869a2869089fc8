"""CPU checker ("oracle") for the selective-rollout decode path -- TEST INFRASTRUCTURE ONLY.

A plain, slow evaluation of what the GPU path computes, written from the paper's
definitions (Section 3.2 for the signal d_K, Eq. 2 for the gate, Eq. 1 for the
advantage, Appendix C.1 for the gated rollout loop) and from the textbook
definition of a pre-norm GQA/SwiGLU decoder.  It shares no code with the GPU
library and must never be imported by it.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may use it.

The arithmetic lives in sr_oracle.c (double precision; a float build is available
as `load(real="float")`); this module is the ctypes wrapper plus the episode loop.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sr_oracle.c")
_LIBS: dict = {}


def _cpu_tag() -> str:
    """Short tag of this host's instruction-set flags: the library is built with -march=native, so a
    copy built on another machine must not be loaded here."""
    import hashlib
    flags = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("flags"):
                flags = line
                break
    except OSError:
        pass
    return hashlib.sha1(flags.encode()).hexdigest()[:8]


# SRO_SANITIZE=1 in the environment: every load() in this process takes the build instrumented with
# AddressSanitizer and UndefinedBehaviorSanitizer (the process must have been started with the sanitizer
# runtime preloaded; tests/test_oracle_sanitized.py does that for a child process).
_SANITIZE = os.environ.get("SRO_SANITIZE", "") == "1"


def _lib_path(real: str, sanitize: bool = False) -> str:
    return os.path.join(_HERE, f"libsroracle_{real}{'_san' if sanitize else ''}_{_cpu_tag()}.so")


def build(force: bool = False, sanitize: bool = False) -> None:
    """Compile sr_oracle.c (double and float builds).  sanitize=True: the double build with
    -fsanitize=address,undefined at -O1 (out-of-bounds accesses, use after free, signed overflow,
    misaligned or null dereferences abort the process), for the host-side sanitizer leg of the tests."""
    for real in (("double",) if sanitize else ("double", "float")):
        out = _lib_path(real, sanitize)
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
            opt = (["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all"] if sanitize else ["-O3", "-march=native"])
            subprocess.check_call(["gcc"] + opt + ["-fopenmp", "-fPIC", "-shared", "-std=c11",
                                   f"-DSRO_REAL={real}", "-o", out, _SRC, "-lm"])


def sanitizer_runtime() -> str:
    """Path of the AddressSanitizer runtime that a process loading the sanitized build must preload."""
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab", "qkv_bias")] + \
               [("rms_eps", ctypes.c_double), ("rope_theta", ctypes.c_double)]


def load(real: str = "double"):
    if real not in _LIBS:
        build(sanitize=_SANITIZE and real == "double")
        L = ctypes.CDLL(_lib_path(real, _SANITIZE and real == "double"))
        vp, ci, cd = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        L.sro_lev.restype = ci
        L.sro_lev.argtypes = [vp, ci, vp, ci]
        L.sro_pair_sum.restype = ctypes.c_int64
        L.sro_pair_sum.argtypes = [vp, ci, ci, ci]
        L.sro_gate_bound.restype = ctypes.c_int64
        L.sro_gate_bound.argtypes = [cd, ci, ci]
        L.sro_mean_prefix_distance.restype = cd
        L.sro_mean_prefix_distance.argtypes = [vp, ci, ci, ci]
        L.sro_gate_batch.restype = None
        L.sro_gate_batch.argtypes = [vp, ci, ci, ci, vp, ci, cd, vp, vp]
        L.sro_advantage.restype = None
        L.sro_advantage.argtypes = [vp, ci, cd, vp]
        L.sro_logprob.restype = cd
        L.sro_logprob.argtypes = [vp, ci, ctypes.c_int32]
        L.sro_grpo_loss.restype = cd
        L.sro_grpo_loss.argtypes = [vp, vp, ci, ci, cd, vp]
        L.sro_signals_batch.restype = None
        L.sro_signals_batch.argtypes = [vp, vp, vp, ci, ci, ci, vp, ci, cd, cd, vp]
        L.sro_lcm32.restype = ctypes.c_int64
        L.sro_model_new.restype = vp
        L.sro_model_new.argtypes = [ctypes.POINTER(_Shape), vp, vp, vp]
        L.sro_model_set_layer.restype = None
        L.sro_model_set_layer.argtypes = [vp, ci] + [vp] * 12
        L.sro_model_free.restype = None
        L.sro_model_free.argtypes = [vp]
        L.sro_seq_new.restype = vp
        L.sro_seq_new.argtypes = [vp, ci]
        L.sro_seq_free.restype = None
        L.sro_seq_free.argtypes = [vp]
        L.sro_seq_len.restype = ci
        L.sro_seq_len.argtypes = [vp]
        L.sro_seq_truncate.restype = None
        L.sro_seq_truncate.argtypes = [vp, ci]
        L.sro_seq_clone.restype = vp
        L.sro_seq_clone.argtypes = [vp, vp]
        L.sro_bf16_round.restype = cd
        L.sro_bf16_round.argtypes = [cd]
        L.sro_forward_token.restype = ci
        L.sro_forward_token.argtypes = [vp, vp, ctypes.c_int32, vp]
        L.sro_forward.restype = ci
        L.sro_forward.argtypes = [vp, vp, vp, ci, vp]
        L.sro_argmax.restype = ci
        L.sro_argmax.argtypes = [vp, ci, ctypes.POINTER(cd)]
        L.sro_sample.restype = ci
        L.sro_sample.argtypes = [vp, ci, cd, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(cd)]
        L.sro_real_bytes.restype = ci
        L.sro_set_bf16_contract.restype = None
        L.sro_set_bf16_contract.argtypes = [ci]
        L.sro_rope_apply.restype = None
        L.sro_rope_apply.argtypes = [vp, ci, ci, cd]
        _LIBS[real] = L
    return _LIBS[real]


# ----------------------------------------------------------------------------
# gate
# ----------------------------------------------------------------------------
def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def lev(a, b) -> int:
    a, b = _i32(a), _i32(b)
    return load().sro_lev(a.ctypes.data, len(a), b.ctypes.data, len(b))


def pair_sum(actions, K: int) -> int:
    """S_K for one group; actions is [G, >=K]."""
    a = _i32(actions)
    return int(load().sro_pair_sum(a.ctypes.data, a.shape[0], a.shape[1], K))


def gate_bound(d_L: float, G: int, K: int) -> int:
    """Smallest integer T with: d_K < d_L  <=>  S_K < T  (Eq. 2 in integers)."""
    return int(load().sro_gate_bound(d_L, G, K))


def mean_prefix_distance(actions, K: int) -> float:
    a = _i32(actions)
    return float(load().sro_mean_prefix_distance(a.ctypes.data, a.shape[0], a.shape[1], K))


def gate_batch(actions, lens, d_L: float):
    """actions [n_groups, G, stride] -> (sums int32 [n_lens, n_groups], cut uint8 [n_lens, n_groups])."""
    a = _i32(actions)
    n_groups, G, stride = a.shape
    lens = _i32(lens)
    sums = np.zeros((len(lens), n_groups), dtype=np.int32)
    cut = np.zeros((len(lens), n_groups), dtype=np.uint8)
    load().sro_gate_batch(a.ctypes.data, n_groups, G, stride, lens.ctypes.data, len(lens), d_L,
                          sums.ctypes.data, cut.ctypes.data)
    return sums, cut


SIGNALS_DTYPE = np.dtype([("d_K", "f8"), ("lev_scaled", "i8"), ("bigram_jaccard", "f8"), ("action_entropy", "f8"),
                          ("unique_prefix", "i4"), ("n_at_step", "i4"), ("unique_action", "i4"), ("unique_obs", "i4"),
                          ("n_done", "i4"), ("lev_sum", "i4"), ("cut_d", "u1"), ("cut_or", "u1")], align=True)


def lcm32() -> int:
    """lcm(1..32): lev_scaled / lcm32() is the exact sum over pairs of lev / longer length."""
    return int(load().sro_lcm32())


def signals_batch(actions, lens, d_L: float, tau_H: float = 2.0, obs=None, end_step=None) -> np.ndarray:
    """Appendix B signals and the gates of Eq. 2 / Eq. 3 at each step K in `lens`.

    actions, obs: [n_groups, G, stride] ids; end_step: [n_groups, G] number of steps after which a member
    finished (anything > stride while it is still running).  Returns a structured array [n_lens, n_groups].
    """
    a = _i32(actions)
    n_groups, G, stride = a.shape
    lens = _i32(lens)
    o = _i32(obs) if obs is not None else None
    e = _i32(end_step) if end_step is not None else None
    out = np.zeros((len(lens), n_groups), dtype=SIGNALS_DTYPE)
    assert SIGNALS_DTYPE.itemsize == 64
    load().sro_signals_batch(a.ctypes.data, o.ctypes.data if o is not None else None,
                             e.ctypes.data if e is not None else None, n_groups, G, stride, lens.ctypes.data,
                             len(lens), d_L, tau_H, out.ctypes.data)
    return out


def advantage(r, eps: float = 1e-6) -> np.ndarray:
    r = np.ascontiguousarray(r, dtype=np.float64)
    A = np.empty_like(r)
    load().sro_advantage(r.ctypes.data, len(r), eps, A.ctypes.data)
    return A


# ----------------------------------------------------------------------------
# decoder
# ----------------------------------------------------------------------------
class Model:
    """Borrowed bf16 weights (uint16 numpy arrays, kept alive here) behind the C decoder."""

    def __init__(self, weights, real: str = "double", n_layers: int | None = None):
        self.L = load(real)
        self.real = np.float64 if real == "double" else np.float32
        self.w = weights
        s = weights.shape
        nl = len(weights.layers) if n_layers is None else n_layers
        self.shape = s
        self.n_layers = nl
        sh = _Shape(nl, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn, s.vocab, int(s.qkv_bias),
                    s.rms_eps, s.rope_theta)
        self.h = self.L.sro_model_new(ctypes.byref(sh), weights.embed.ctypes.data, weights.lm_head.ctypes.data,
                                      weights.final_norm.ctypes.data)
        order = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "bq", "bk", "bv", "norm1", "norm2")
        for l in range(nl):
            d = weights.layers[l]
            self.L.sro_model_set_layer(self.h, l, *[d[k].ctypes.data for k in order])

    def __del__(self):
        try:
            self.L.sro_model_free(self.h)
        except Exception:
            pass

    def new_seq(self, cap: int) -> "Seq":
        return Seq(self, cap)


class Seq:
    def __init__(self, model: Model, cap: int, _handle=None):
        self.m = model
        self.h = model.L.sro_seq_new(model.h, cap) if _handle is None else _handle

    def clone(self) -> "Seq":
        """An independent sequence with the same tokens behind it (e.g. the G members of a group after their
        common prompt: sequences do not interact, so evaluating the prompt once and copying is exact)."""
        return Seq(self.m, 0, _handle=self.m.L.sro_seq_clone(self.m.h, self.h))

    def __del__(self):
        try:
            self.m.L.sro_seq_free(self.h)
        except Exception:
            pass

    def __len__(self):
        return self.m.L.sro_seq_len(self.h)

    def truncate(self, n: int):
        self.m.L.sro_seq_truncate(self.h, n)

    def forward(self, tokens, want_logits: bool = True):
        """Append tokens; returns the logits after the last one (or None)."""
        t = _i32(np.atleast_1d(tokens))
        out = np.empty(self.m.shape.vocab, dtype=self.m.real) if want_logits else None
        rc = self.m.L.sro_forward(self.m.h, self.h, t.ctypes.data, len(t),
                                  out.ctypes.data if want_logits else None)
        if rc:
            raise RuntimeError("oracle sequence capacity exceeded")
        return out


def set_bf16_contract(on: bool, real: str = "double") -> None:
    """Round activations to bf16 where a bf16 tensor-core implementation must (see sr_oracle.c).
    Off by default; the exact evaluation is the reference, this mode only attributes error."""
    load(real).sro_set_bf16_contract(int(on))


def bf16_round(x: float) -> float:
    """The contract mode's rounding of one value: to single precision, then to the nearest bf16, ties to even."""
    return float(load().sro_bf16_round(float(x)))


def rope_apply(vec, pos: int, theta: float) -> np.ndarray:
    """Rotate one head vector (fp64) to absolute position pos."""
    v = np.array(vec, dtype=np.float64)
    load().sro_rope_apply(v.ctypes.data, len(v), pos, theta)
    return v


def argmax(logits):
    """(lowest index among maxima, gap between the best and second-best logit)."""
    lg = np.ascontiguousarray(logits)
    L = load("double" if lg.dtype == np.float64 else "float")
    gap = ctypes.c_double()
    idx = L.sro_argmax(lg.ctypes.data, len(lg), ctypes.byref(gap))
    return idx, gap.value


def sample(logits, temperature: float, seed: int, orig_seq: int, pos: int):
    """(token drawn from softmax(logits / T) by the Gumbel-max rule with counter-based uniforms keyed
    (seed, original sequence id, position); gap between the best and second-best perturbed score)."""
    lg = np.ascontiguousarray(logits)
    L = load("double" if lg.dtype == np.float64 else "float")
    gap = ctypes.c_double()
    idx = L.sro_sample(lg.ctypes.data, len(lg), temperature, seed, orig_seq, pos, ctypes.byref(gap))
    return idx, gap.value


# ----------------------------------------------------------------------------
# gated group rollout (Appendix C.1)
# ----------------------------------------------------------------------------
def logprob(logits, target: int) -> float:
    """log softmax(logits)[target] (logits as returned by Seq.forward)."""
    lg = np.ascontiguousarray(logits)
    real = "float" if lg.dtype == np.float32 else "double"
    return float(load(real).sro_logprob(lg.ctypes.data, len(lg), int(target)))


def score(seq: "Seq", last_logits, tokens, mask=None):
    """Teacher-forced pass over `tokens` appended to `seq` (Appendix C.2).

    last_logits: logits at the sequence's current last position (they predict tokens[0]).
    Returns (per-token log-probabilities, with 0 where mask is 0; logits at the new last position).
    """
    tokens = _i32(tokens)
    lp = np.zeros(len(tokens))
    logits = last_logits
    for j, tok in enumerate(tokens):
        if mask is None or mask[j]:
            lp[j] = logprob(logits, tok)
        logits = seq.forward([tok])
    return lp, logits


def grpo_loss(logprob_seq, rewards, G: int, eps: float = 1e-6):
    """(-(1/N) sum_i A_i log p(tau_i), advantages) for [n_groups*G] sequence log-likelihoods and rewards."""
    lp = np.ascontiguousarray(logprob_seq, dtype=np.float64)
    r = np.ascontiguousarray(rewards, dtype=np.float64)
    A = np.empty_like(r)
    loss = load().sro_grpo_loss(lp.ctypes.data, r.ctypes.data, len(r) // G, G, eps, A.ctypes.data)
    return float(loss), A


def run_episode(model: Model, prompts, obs_fn, G: int, turns: int, act_len: int, action_mod: int,
                gate_turns, d_L: float, keep_logits: bool = False, temperature: float = 0.0, sample_seed: int = 0,
                finish_fn=None, tau_H: float | None = None):
    """Rolls every group forward turn by turn, gating at the given turns.

    prompts: int32 [n_groups, P] (shared by the G members of a group).
    obs_fn(turn) -> int32 [n_groups*G, obs_len] rows in ORIGINAL (group-major) order.
    Each turn appends the observation chunk, then decodes act_len tokens (greedily, or sampled at
    `temperature` > 0 with `sample` keyed by the sequence's original id and its current length); the
    turn's action id is (first decoded token) mod action_mod.  After a gate turn K the
    pairwise-distance sum S_K over the first K actions is compared with gate_bound and
    groups with S_K < bound stop there and leave the batch.

    finish_fn(K, r) -> bool (optional): sequence r's trajectory ends after environment step K (reported by the
    environment, i.e. an input here); it generates nothing further, its group goes on with the other members,
    and a group whose last member ends leaves the batch without being cut.  With finish_fn the gate compares
    prefixes of unequal length (each pair divided by the longer one) and, if tau_H is given, also cuts a group
    when the fraction of its members that have ended is >= tau_H (Appendix E, Eq. 3).

    Returns a dict of per-turn records, all indexed by original sequence / group ids.
    """
    prompts = _i32(prompts)
    n_groups, P = prompts.shape
    n_seq = n_groups * G
    obs0 = obs_fn(0)
    cap = P + turns * (obs0.shape[1] + act_len)
    seqs = [None] * n_seq
    live = list(range(n_groups))
    actions = np.full((n_seq, turns), -1, dtype=np.int32)
    alive = np.ones(n_seq, dtype=bool)
    end_step = np.full(n_seq, 10 ** 6, dtype=np.int32)
    rec = {"tokens": [], "gaps": [], "logits": [], "live_groups": [], "live_rows": [], "finished": [], "gate": {},
           "decoded_tokens": 0}

    # the prompt is common to the G members of a group and sequences do not interact: evaluate it once per
    # group and copy the resulting sequence state for the other members
    logits = [None] * n_seq
    for g in live:
        first = model.new_seq(cap)
        lg = first.forward(prompts[g])
        for m in range(G):
            seqs[g * G + m] = first if m == 0 else first.clone()
            logits[g * G + m] = lg if m == 0 else lg.copy()

    for turn in range(turns):
        obs = obs0 if turn == 0 else obs_fn(turn)
        rows = [g * G + m for g in live for m in range(G) if alive[g * G + m]]
        rec["live_groups"].append(list(live))
        rec["live_rows"].append(list(rows))
        for r in rows:
            logits[r] = seqs[r].forward(obs[r])
        t_tok = np.full((act_len, n_seq), -1, dtype=np.int32)
        t_gap = np.full((act_len, n_seq), np.inf)
        t_log = []
        for a in range(act_len):
            if keep_logits:
                t_log.append({r: logits[r].copy() for r in rows})
            for r in rows:
                if temperature > 0:
                    tok, gap = sample(logits[r], temperature, sample_seed, r, len(seqs[r]))
                else:
                    tok, gap = argmax(logits[r])
                t_tok[a, r], t_gap[a, r] = tok, gap
                if a == 0:
                    actions[r, turn] = tok % action_mod
                logits[r] = seqs[r].forward([tok])
                rec["decoded_tokens"] += 1
        rec["tokens"].append(t_tok)
        rec["gaps"].append(t_gap)
        rec["logits"].append(t_log)
        K = turn + 1
        done_now = [r for r in rows if finish_fn is not None and finish_fn(K, r)]
        for r in done_now:
            alive[r] = False
            end_step[r] = K
        rec["finished"].append(done_now)
        live = [g for g in live if alive[g * G:(g + 1) * G].any()]
        if K in gate_turns:
            if finish_fn is None:
                bound = gate_bound(d_L, G, K)
                sums = {g: pair_sum(actions[g * G:(g + 1) * G], K) for g in live}
                cut = {g: sums[g] < bound for g in live}
                rec["gate"][K] = {"bound": bound, "sums": sums, "cut": cut}
            elif live:
                sig = signals_batch(np.stack([actions[g * G:(g + 1) * G] for g in live]), [K], d_L,
                                    2.0 if tau_H is None else tau_H,
                                    end_step=np.stack([end_step[g * G:(g + 1) * G] for g in live]))[0]
                key = "cut_d" if tau_H is None else "cut_or"
                rec["gate"][K] = {"sums": {g: int(sig["lev_sum"][i]) for i, g in enumerate(live)},
                                  "cut": {g: bool(sig[key][i]) for i, g in enumerate(live)},
                                  "n_done": {g: int(sig["n_done"][i]) for i, g in enumerate(live)}}
            else:
                rec["gate"][K] = {"sums": {}, "cut": {}, "n_done": {}}
            cut = rec["gate"][K]["cut"]
            live = [g for g in live if not cut[g]]
    rec["actions"] = actions
    rec["end_step"] = end_step
    rec["final_live_groups"] = live
    return rec
