"""Glue used by the tests, the smoke entry and the benchmark: moves seeded synthetic weights and
batches to the GPU and calls the binding.  No arithmetic of the method lives here."""
from __future__ import annotations

from typing import Dict, Optional, Tuple

import numpy as np
import torch

from . import binding, synth


def _to_dev(a: np.ndarray, dtype: torch.dtype, device: str) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).to(device)


def upload_model(weights: synth.SynthWeights, device: str = "cuda", lm_head=None, compute_dtype: Optional[str] = None,
                 hilo_layers: int = 0, lm_head_mode: int = 0, fold_norms: int = 0) -> binding.Model:
    """Generate the weights layer by layer, copy them to the GPU and create the library model
    (which keeps its own re-packed copy, so the uploaded tensors are released afterwards).
    compute_dtype / hilo_layers / lm_head_mode / fold_norms are the library-side settings of radix_model_config
    (operand type, leading layers with (hi, lo) GEMM inputs, LM head, RMSNorms folded into the GEMMs); lm_head: the separate head matrix
    for lm_head_mode 2."""
    cfg = weights.cfg
    mt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    embed = _to_dev(weights.embed, mt, device)
    gf = _to_dev(weights.gf, torch.float32, device)
    layers = []
    for l in range(cfg.n_layers):
        lw = weights.layer(l)
        layers.append({k: _to_dev(v, torch.float32 if k.startswith("g") else mt, device) for k, v in lw.items()})
    head = None if lm_head is None else _to_dev(lm_head, mt, device)      # only read when lm_head_mode == 2
    model = binding.radix_model_create(cfg, embed, gf, layers, lm_head=head, compute_dtype=compute_dtype,
                                       hilo_layers=hilo_layers, lm_head_mode=lm_head_mode, fold_norms=fold_norms)
    torch.cuda.synchronize()
    return model


def upload_batch(batch: synth.Batch, device: str = "cuda") -> Tuple[torch.Tensor, torch.Tensor]:
    tok = torch.from_numpy(batch.tok.astype(np.int32)).to(device)
    cu = torch.from_numpy(batch.cu_seqlens.astype(np.int32)).to(device)
    return tok, cu


class Runner:
    """A model, a workspace sized for one batch shape, and the three calls of the path."""

    def __init__(self, model: binding.Model, max_N: int, max_B: int):
        self.model = model
        self.ws = binding.alloc_workspace(binding.radix_workspace_bytes(model, max_N, max_B))

    def build_index(self, tok, cu, pos=None):
        return binding.radix_build_index(tok, pos, cu, self.ws)

    def forward(self, tok, cu, max_seqlen, maps, pos=None, out=None, **kw):
        I_s, I_g, _, n_c = maps
        return binding.radix_prefill_forward(self.model, tok, pos, cu, max_seqlen, I_s, I_g, n_c, self.ws, out=out, **kw)

    def forward_nodedup(self, tok, cu, max_seqlen, pos=None, out=None):
        return binding.radix_prefill_forward_nodedup(self.model, tok, pos, cu, max_seqlen, self.ws, out=out)

    def status(self) -> int:
        return binding.radix_device_status(self.ws)
