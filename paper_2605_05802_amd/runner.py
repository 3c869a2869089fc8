"""Episode driver on top of the C boundary: uploads weights and walks the turn loop.

Marshalling and control flow only (which call comes next); every number is produced by libsr.so.
"""
from __future__ import annotations

import numpy as np
import torch

from . import Context


def upload_bits(a: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns -> int16 device tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device)


def load_host_weights(ctx: Context, w, n_layers=None):
    """Upload synth.HostWeights and hand them to sr_load_weights (the library keeps its own packed copy)."""
    L = len(w.layers) if n_layers is None else n_layers
    embed, lm, fn = upload_bits(w.embed), upload_bits(w.lm_head), upload_bits(w.final_norm)
    layers = [{k: upload_bits(v) for k, v in w.layers[l].items()} for l in range(L)]
    ctx.sr_load_weights(embed, lm, fn, layers)
    torch.cuda.synchronize()


class Episode:
    """One gated rollout: prompt prefill, then per turn an observation chunk and act_len decode steps."""

    def __init__(self, ctx: Context, G: int, act_len: int, gate_turns=()):
        self.ctx, self.G, self.act_len, self.gate_turns = ctx, G, act_len, tuple(gate_turns)
        self.turn = 0

    def prefill_prompt(self, prompts_dev):
        self.ctx.sr_prefill_chunk(prompts_dev, True)

    def run_turn(self, obs_dev, forced=None, out_tokens=None):
        """obs_dev: int32 [n_live_seq, obs_len] on the device.  forced/out_tokens: optional lists of
        act_len device tensors.  Returns the number of live groups after the (possible) gate."""
        self.ctx.sr_prefill_chunk(obs_dev, False)
        for a in range(self.act_len):
            self.ctx.sr_decode_step(None if forced is None else forced[a],
                                    None if out_tokens is None else out_tokens[a])
        self.turn += 1
        if self.turn in self.gate_turns:
            self.ctx.sr_gate(self.turn)
            return self.ctx.sr_retire_and_compact()
        return None
