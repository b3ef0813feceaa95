"""Where the 16-bit path spends its error budget, reproduced on the CPU from the oracle's own functions.

The HIP path rounds activations to the 16-bit operand type at six points per layer: the two RMSNorm outputs
(a, b), q/k after Q/K-norm + RoPE, v, the attention output (o) and the SwiGLU output (m).  Everything else is
fp32.  This file re-runs the oracle's forward in fp64 with exactly those roundings inserted (nothing of the HIP
path is involved) and checks the three statements the library's precision settings rest on:

  1. bf16 operands (8-bit significands) cost about 0.6 % RMS / 3e-2 max on the 28-layer 0.6B shape: above the
     2e-2 bar, which is why fp16 operands (11 bits) are the default and bf16 operands carry no parity claim;
  2. on a deep model whose projections do not attenuate (gain rms(W) sqrt(d) >= 1), most of the final error is
     made in layer 0, whose outputs are the whole residual stream at that depth;
  3. carrying all six points of layer 0 as (hi, lo) pairs removes more than half of the error for 1 / n_layers more
     GEMM work (the automatic hilo_layers setting); the four GEMM inputs (a, b, o, m) alone, even in two layers,
     remove about a third.
"""
import dataclasses
import math

import numpy as np
import torch

from oracle import forward as orc
from paper_2601_15013_amd import synth

POINTS = ("a", "qk", "v", "o", "b", "m")


def _round(x, mode):
    """mode: None (exact), "bf16", "f16", or "f16x2" = a (hi, lo) pair of fp16 values."""
    if mode is None:
        return x
    if mode == "bf16":
        return x.bfloat16().double()
    hi = x.half().double()
    if mode == "f16":
        return hi
    return hi + (x - hi).half().double()


def _forward(cfg, embed_rows, layers, gf, modes_of_layer):
    """The oracle's layer sequence for ONE sequence with a rounding mode per point and layer."""
    x = torch.from_numpy(embed_rows).double()
    n = x.shape[0]
    p = torch.arange(n)
    hq, hkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    for l, w in enumerate(layers):
        m = modes_of_layer(l)
        a = _round(orc.rmsnorm(x, w["g1"], cfg.eps), m["a"])
        q = (a @ w["wq"].T).reshape(n, hq, hd)
        k = (a @ w["wk"].T).reshape(n, hkv, hd)
        v = _round(a @ w["wv"].T, m["v"]).reshape(n, hkv, hd)
        q = _round(orc.rope(orc.rmsnorm(q, w["gq"], cfg.eps), p, cfg.rope_base), m["qk"])
        k = _round(orc.rope(orc.rmsnorm(k, w["gk"], cfg.eps), p, cfg.rope_base), m["qk"])
        o = _round(orc.causal_attention(q, k, v).reshape(n, hq * hd), m["o"])
        x = x + o @ w["wo"].T
        b = _round(orc.rmsnorm(x, w["g2"], cfg.eps), m["b"])
        x = x + _round(orc.silu(b @ w["wg"].T) * (b @ w["wu"].T), m["m"]) @ w["wd"].T
    return orc.rmsnorm(x, torch.from_numpy(gf).double(), cfg.eps).numpy()


class _Case:
    def __init__(self, cfg, seed, batch, sequences, scale=1.0):
        self.cfg = cfg
        w = synth.SynthWeights(cfg, seed)
        self.layers = []
        for l in range(cfg.n_layers):
            self.layers.append({k: torch.from_numpy(v * scale if not k.startswith("g") else v).double()
                                for k, v in w.layer(l).items()})
        self.gf = w.gf
        emb = w.embed
        cu = batch.cu_seqlens
        self.rows = [emb[batch.tok[cu[s]:cu[s + 1]]] for s in sequences]
        self.ref = self.run(lambda l: dict.fromkeys(POINTS))
        self.rms = math.sqrt(float(np.mean(self.ref ** 2)))

    def run(self, modes_of_layer):
        return np.concatenate([_forward(self.cfg, r, self.layers, self.gf, modes_of_layer) for r in self.rows])

    def err(self, modes_of_layer):
        e = np.abs(self.run(modes_of_layer) - self.ref)
        return float(e.max()) / self.rms, math.sqrt(float(np.mean(e ** 2))) / self.rms


def test_exact_modes_reproduce_the_oracle():
    cfg = dataclasses.replace(synth.QWEN3_0_6B, n_layers=2, vocab=4096)
    b = synth.shared_prefix_batch(5, 2, 4, 3, 9, cfg.vocab)
    case = _Case(cfg, 91, b, [0, 1])
    w = synth.SynthWeights(cfg, 91)
    want = orc.forward_nodedup(cfg, w.embed, w.layers, w.gf, b.tok, b.cu_seqlens)
    assert np.array_equal(case.ref, want)


def test_bf16_operands_exceed_the_bar_and_fp16_operands_do_not():
    b = synth.make_batch("C2")
    case = _Case(synth.QWEN3_0_6B, synth.WORKLOADS["C2"].seed, b, [0, 17])
    mx_b, rms_b = case.err(lambda l: dict.fromkeys(POINTS, "bf16"))
    mx_h, rms_h = case.err(lambda l: dict.fromkeys(POINTS, "f16"))
    print(f"0.6B shape, 28 layers: bf16 roundings max {mx_b:.3e} rms {rms_b:.3e}; fp16 roundings max {mx_h:.3e} rms {rms_h:.3e}")
    assert 2e-2 < mx_b < 6e-2 and 3.5e-3 < rms_b < 9e-3
    assert mx_h < 8e-3 and rms_h < rms_b / 6.0          # three more bits: 8x smaller


def test_first_layers_dominate_and_hilo_inputs_there_pay():
    # the 0.6B shape with weights scaled x2 (sigma 0.04, gain 0.04 * sqrt(1024) = 1.28) and 36 layers behaves like the
    # 8B shape (gain 0.02 * sqrt(4096) = 1.28) at a size the CPU handles in seconds
    cfg = dataclasses.replace(synth.QWEN3_0_6B, n_layers=36)
    b = synth.make_batch("C2")
    case = _Case(cfg, 77, b, [0, 17, 33], scale=2.0)
    f16 = dict.fromkeys(POINTS, "f16")
    exact = dict.fromkeys(POINTS)
    hilo = dict(f16, a="f16x2", b="f16x2", o="f16x2", m="f16x2")
    hilo6 = dict.fromkeys(POINTS, "f16x2")
    mx_all, rms_all = case.err(lambda l: f16)
    mx_l0, rms_l0 = case.err(lambda l: f16 if l == 0 else exact)
    mx_rest, rms_rest = case.err(lambda l: exact if l == 0 else f16)
    mx_h2, rms_h2 = case.err(lambda l: hilo if l < 2 else f16)
    mx_hall, rms_hall = case.err(lambda l: hilo)
    mx_6, rms_6 = case.err(lambda l: hilo6 if l == 0 else f16)
    print(f"gain-1.28 proxy, 36 layers, fp16 roundings: all layers rms {rms_all:.3e} (max {mx_all:.3e}); layer 0 only "
          f"{rms_l0:.3e}; all but layer 0 {rms_rest:.3e}; (hi, lo) a/b/o/m in layers 0-1 {rms_h2:.3e} (max {mx_h2:.3e}); "
          f"in all layers {rms_hall:.3e}; all six points (hi, lo) in layer 0 {rms_6:.3e} (max {mx_6:.3e})")
    assert rms_l0 > 0.75 * rms_all                  # layer 0 alone makes most of the error ...
    assert rms_rest < 0.65 * rms_all                # ... and the other 35 layers together much less
    assert rms_h2 < 0.75 * rms_all                  # two (hi, lo) layers: a third of the error gone
    assert rms_h2 < 1.25 * rms_hall                 # and most of what (hi, lo) inputs in every layer would give
    assert rms_6 < 0.55 * rms_all                   # all six points in layer 0 alone: more than half of the error gone
