"""Seeded synthetic inputs (weights, prompts, observations, action tables).

Input generation only: nothing here computes an edit distance, a gate decision
or any decoder arithmetic.  The CPU checker and the GPU library both consume
the arrays produced here, so that the two can be compared on identical inputs.

The random stream is SplitMix64 used counter-based (see srsynth.c).  Normal
variates come from a 65536-entry bf16 quantile table built here in fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsrsynth.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile srsynth.c with gcc into libsrsynth.so (next to this file)."""
    src = os.path.join(_HERE, "srsynth.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB_PATH, src])
    return _LIB_PATH


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        u64, sz, vp = ctypes.c_uint64, ctypes.c_size_t, ctypes.c_void_p
        L.srs_stream_key.restype = u64
        L.srs_stream_key.argtypes = [u64, u64]
        L.srs_draw.restype = u64
        L.srs_draw.argtypes = [u64, u64]
        L.srs_fill_table16.restype = None
        L.srs_fill_table16.argtypes = [vp, sz, u64, u64, u64, vp]
        L.srs_fill_ids.restype = None
        L.srs_fill_ids.argtypes = [vp, sz, u64, u64, ctypes.c_uint32]
        L.srs_gate_actions.restype = None
        L.srs_gate_actions.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       vp, ctypes.c_int, u64, vp]
        _lib = L
    return _lib


# ----------------------------------------------------------------------------
# bf16 helpers (storage format only)
# ----------------------------------------------------------------------------
def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp64 -> fp32 -> bf16 (round to nearest even), returned as uint16 bit patterns."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


_TABLES: dict = {}


def normal_table(sigma: float) -> np.ndarray:
    """65536 quantiles of N(0, sigma) at probabilities (j + 0.5) / 65536, as bf16 bits."""
    if sigma not in _TABLES:
        from scipy.special import ndtri
        p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
        _TABLES[sigma] = np.ascontiguousarray(f64_to_bf16_bits(sigma * ndtri(p)))
    return _TABLES[sigma]


# ----------------------------------------------------------------------------
# model shape and weight tensors
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    qkv_bias: bool = True

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim


TINY = ModelShape(2, 256, 4, 2, 64, 688, 1024)
QWEN7B = ModelShape(28, 3584, 28, 4, 128, 18944, 152064)

# stream ids of the weight tensors
STREAM_EMBED, STREAM_LM_HEAD = 1, 2
_LAYER_SLOTS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "bq", "bk", "bv")


def layer_stream(layer: int, name: str) -> int:
    return 16 * (layer + 1) + _LAYER_SLOTS.index(name)


def tensor_shapes(s: ModelShape) -> dict:
    """name -> shape of every per-layer tensor; matrices are [out_features, in_features]."""
    return {
        "wq": (s.q_dim, s.hidden), "wk": (s.kv_dim, s.hidden), "wv": (s.kv_dim, s.hidden),
        "wo": (s.hidden, s.q_dim), "wg": (s.ffn, s.hidden), "wu": (s.ffn, s.hidden),
        "wd": (s.hidden, s.ffn), "bq": (s.q_dim,), "bk": (s.kv_dim,), "bv": (s.kv_dim,),
    }


def fill_normal_bf16(n: int, seed: int, stream: int, sigma: float = 0.02, first: int = 0) -> np.ndarray:
    out = np.empty(n, dtype=np.uint16)
    tab = normal_table(sigma)
    lib().srs_fill_table16(out.ctypes.data, n, seed, stream, first, tab.ctypes.data)
    return out


@dataclass
class HostWeights:
    """bf16 bit patterns (uint16 numpy arrays).  Norm gains are 1.0."""
    shape: ModelShape
    embed: np.ndarray
    lm_head: np.ndarray
    final_norm: np.ndarray
    layers: list = field(default_factory=list)   # list of dict name -> array (+ "norm1", "norm2")


def make_weights(s: ModelShape, seed: int = 0, sigma: float = 0.02, n_layers: int | None = None) -> HostWeights:
    """All matrices and biases N(0, sigma) as bf16; RMSNorm gains 1.0 (bf16 0x3F80)."""
    L = s.n_layers if n_layers is None else n_layers
    one = np.uint16(0x3F80)
    w = HostWeights(
        shape=s,
        embed=fill_normal_bf16(s.vocab * s.hidden, seed, STREAM_EMBED, sigma).reshape(s.vocab, s.hidden),
        lm_head=fill_normal_bf16(s.vocab * s.hidden, seed, STREAM_LM_HEAD, sigma).reshape(s.vocab, s.hidden),
        final_norm=np.full(s.hidden, one, dtype=np.uint16),
    )
    shapes = tensor_shapes(s)
    for l in range(L):
        d = {}
        for name, shp in shapes.items():
            n = int(np.prod(shp))
            if name in ("bq", "bk", "bv") and not s.qkv_bias:
                d[name] = np.zeros(shp, dtype=np.uint16)
            else:
                d[name] = fill_normal_bf16(n, seed, layer_stream(l, name), sigma).reshape(shp)
        d["norm1"] = np.full(s.hidden, one, dtype=np.uint16)
        d["norm2"] = np.full(s.hidden, one, dtype=np.uint16)
        w.layers.append(d)
    return w


# ----------------------------------------------------------------------------
# device-side weight fill (same stream, same table; for multi-gigabyte models)
# ----------------------------------------------------------------------------
_HIP_LIB_PATH = os.path.join(_HERE, "libsrsynth_hip.so")
_hip_lib = None


def build_hip(force: bool = False) -> str:
    src = os.path.join(_HERE, "srsynth_hip.hip")
    if force or not os.path.exists(_HIP_LIB_PATH) or os.path.getmtime(_HIP_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O2", "-fPIC", "-shared",
                               "-o", _HIP_LIB_PATH, src])
    return _HIP_LIB_PATH


def hip_lib():
    global _hip_lib
    if _hip_lib is None:
        if not os.path.exists(_HIP_LIB_PATH):
            build_hip()
        L = ctypes.CDLL(_HIP_LIB_PATH)
        L.srs_fill_table16_dev.restype = ctypes.c_int
        L.srs_fill_table16_dev.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_uint64,
                                           ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]
        _hip_lib = L
    return _hip_lib


def make_weights_device(s: ModelShape, seed: int = 0, sigma: float = 0.02, n_layers: int | None = None):
    """The tensors of make_weights, generated directly in HBM (torch int16 tensors holding bf16 bits).

    Returns (embed, lm_head, final_norm, layers) with layers a list of dicts, bit-identical to
    make_weights(...) on the host.
    """
    import torch
    L = s.n_layers if n_layers is None else n_layers
    table = torch.from_numpy(normal_table(sigma).view(np.int16)).cuda()
    stream = torch.cuda.current_stream().cuda_stream

    def fill(shape, stream_id):
        t = torch.empty(shape, dtype=torch.int16, device="cuda")
        rc = hip_lib().srs_fill_table16_dev(t.data_ptr(), t.numel(), seed, stream_id, 0, table.data_ptr(), stream)
        if rc != 0:
            raise RuntimeError(f"device fill failed with HIP error {rc}")
        return t

    ones = lambda n: torch.full((n,), 0x3F80, dtype=torch.int16, device="cuda")
    embed = fill((s.vocab, s.hidden), STREAM_EMBED)
    lm_head = fill((s.vocab, s.hidden), STREAM_LM_HEAD)
    layers = []
    for l in range(L):
        d = {}
        for name, shp in tensor_shapes(s).items():
            if name in ("bq", "bk", "bv") and not s.qkv_bias:
                d[name] = torch.zeros(shp, dtype=torch.int16, device="cuda")
            else:
                d[name] = fill(shp, layer_stream(l, name))
        d["norm1"], d["norm2"] = ones(s.hidden), ones(s.hidden)
        layers.append(d)
    torch.cuda.synchronize()
    return embed, lm_head, ones(s.hidden), layers


# ----------------------------------------------------------------------------
# episode inputs: shared prompts, per-turn observation chunks
# ----------------------------------------------------------------------------
def uniform_ids(n: int, seed: int, stream: int, modulus: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    lib().srs_fill_ids(out.ctypes.data, n, seed, stream, modulus)
    return out


@dataclass(frozen=True)
class EpisodeConfig:
    name: str
    n_groups: int
    G: int
    prompt_len: int
    turns: int
    obs_len: int
    act_len: int
    action_mod: int
    gate_turns: tuple
    threshold: float
    converge_frac: float      # fraction of groups whose members receive identical observations


TINY_EPISODE = EpisodeConfig("tiny", 4, 8, 64, 6, 16, 8, 16, (3,), 0.3, 0.5)
C3_EPISODE = EpisodeConfig("7b-g8-16groups", 16, 8, 1024, 20, 64, 32, 64, (10,), 0.3, 0.4)
C4_EPISODE = EpisodeConfig("7b-g8-64groups", 64, 8, 1024, 30, 64, 32, 64, (10,), 0.3, 0.4)
C5_EPISODE = EpisodeConfig("7b-g16-32groups", 32, 16, 4096, 24, 128, 32, 64, (6, 12), 0.25, 0.4)


def converging_groups(cfg: EpisodeConfig, seed: int) -> np.ndarray:
    """Boolean [n_groups]: exactly round(converge_frac * n_groups) groups, a seeded subset.

    Members of a converging group are fed the same observation tokens every turn, so under
    greedy decoding their token streams (hence their action sequences) are identical.
    """
    n_conv = int(round(cfg.converge_frac * cfg.n_groups))
    score = np.array([lib().srs_draw(lib().srs_stream_key(seed, 0x5E1EC7), g) for g in range(cfg.n_groups)],
                     dtype=np.uint64)
    order = np.argsort(score, kind="stable")
    mask = np.zeros(cfg.n_groups, dtype=bool)
    mask[order[:n_conv]] = True
    return mask


def prompts(cfg: EpisodeConfig, vocab: int, seed: int) -> np.ndarray:
    """int32 [n_groups, prompt_len], uniform ids; one prompt per group."""
    return np.stack([uniform_ids(cfg.prompt_len, seed, (1 << 56) | g, vocab) for g in range(cfg.n_groups)])


def observations(cfg: EpisodeConfig, vocab: int, seed: int, turn: int, conv: np.ndarray) -> np.ndarray:
    """int32 [n_groups * G, obs_len] for one turn (rows group-major)."""
    rows = []
    for g in range(cfg.n_groups):
        for m in range(cfg.G):
            who = 0xFFFF if conv[g] else m
            stream = (3 << 56) | (turn << 40) | (g << 16) | who
            rows.append(uniform_ids(cfg.obs_len, seed, stream, vocab))
    return np.stack(rows)


# ----------------------------------------------------------------------------
# gate-only workload
# ----------------------------------------------------------------------------
GATE_COPY_PROBS = (0.5, 0.8, 0.95, 1.0)


def gate_actions(n_groups: int, G: int = 8, length: int = 30, alphabet: int = 64, seed: int = 0,
                 probs=GATE_COPY_PROBS):
    """int32 [n_groups, G, length] noisy copies of a latent leader; also the per-group p index."""
    p_q16 = np.array([int(round(p * 65536)) for p in probs], dtype=np.uint32)
    out = np.empty((n_groups, G, length), dtype=np.int32)
    pidx = np.empty(n_groups, dtype=np.int32)
    lib().srs_gate_actions(out.ctypes.data, n_groups, G, length, alphabet, p_q16.ctypes.data, len(p_q16),
                           seed, pidx.ctypes.data)
    return out, pidx
