"""Weight upload helpers on top of the C boundary (marshalling only; every number is produced by libsr.so)."""
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
