"""Oracle for the prefill forward pass: NO deduplication, every sequence on its own.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Plain PyTorch CPU ops in float64
(``torch.matmul`` is the only library primitive used as a step); no trie, no index maps,
no blocking or fusion.  The paper states that the deduplicated pass is lossless with
respect to the ordinary forward pass (Background, "The Causal Transformer Block";
Limitations, "Numerical differences without batch-invariant kernels"), so the ordinary
pass *is* the definition of what the deduplicated HIP path must produce.

What is computed, per sequence with tokens t_0..t_{n-1} and positions p_i (default i):

  x_i = E[t_i]                                              embedding
  per layer (block structure: Background Eqs. 1-2; operation order: Algorithm 1):
      a   = RMSNorm(x; g1)
      q,k,v = Wq a, Wk a, Wv a                              no bias
      q_h = RMSNorm_hd(q_h; gq),  k_g = RMSNorm_hd(k_g; gk) per head (Qwen3 Q/K norms)
      q_h, k_g = RoPE(q_h, p), RoPE(k_g, p)
      o_{i,h} = sum_{j<=i} softmax_j(q_{i,h} . k_{j,g(h)} / sqrt(hd)) v_{j,g(h)},  g(h) = h // (Hq/Hkv)
      x  += Wo o
      b   = RMSNorm(x; g2)
      x  += Wd ( silu(Wg b) * (Wu b) )                      SwiGLU MLP, Background Eq. 5
  y_i = RMSNorm(x_i; gf)                                    final norm (Algorithm 1, "Output")

Readings where the paper is silent: the paper's "LayerNorm" is
RMSNorm x * rsqrt(mean(x^2) + eps) * g with eps inside the square root; RoPE pairs element i
with i + hd/2, angle p * base^(-2i/hd); softmax scale 1/sqrt(hd); silu(z) = z / (1 + exp(-z));
the output is the final-norm hidden state; ``lm_head_logits`` is Algorithm 1's tail (logits = LMHead(h)) for
the rows a caller selects, with the head tied to the embedding when no separate matrix is given.

Pins (tests/test_oracle_forward.py): a composition of torch's own library routines
(embedding, rms_norm, linear, scaled_dot_product_attention(is_causal), silu, complex-number
rotation for RoPE) on the tiny config; closed forms (single-token sequences, zeroed output
projections, rotation properties of RoPE); invariants (causality, batch independence,
duplicate sequences give duplicate rows).  The paper prints no activation values, so the
values themselves have no printed pin.
"""
from __future__ import annotations

import math
from typing import Any, Iterable, Mapping, Optional, Sequence

import numpy as np
import torch


def _t(a: Any, dtype: torch.dtype) -> torch.Tensor:
    return torch.as_tensor(np.asarray(a)).to(dtype)


def rmsnorm(x: torch.Tensor, g: torch.Tensor, eps: float) -> torch.Tensor:
    """x * rsqrt(mean(x^2) + eps) * g over the last axis."""
    ms = (x * x).sum(dim=-1, keepdim=True) / x.shape[-1]
    return x / torch.sqrt(ms + eps) * g


def rope(x: torch.Tensor, p: torch.Tensor, base: float) -> torch.Tensor:
    """Rotary embedding on x[n, heads, hd]; element i is paired with i + hd/2.

    theta_i = base^(-2i/hd); (x_i, x_{i+hd/2}) is rotated by the angle p * theta_i.
    """
    hd = x.shape[-1]
    half = hd // 2
    i = torch.arange(half, dtype=x.dtype)
    theta = torch.pow(torch.tensor(base, dtype=x.dtype), -2.0 * i / hd)
    ang = p.to(x.dtype)[:, None] * theta[None, :]          # [n, half]
    c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * c - x2 * s, x2 * c + x1 * s], dim=-1)


def causal_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor) -> torch.Tensor:
    """q[n, Hq, hd], k,v[n, Hkv, hd] of ONE sequence -> o[n, Hq, hd]; query i sees keys j <= i."""
    n, hq, hd = q.shape
    hkv = k.shape[1]
    group = hq // hkv
    o = torch.empty_like(q)
    allowed = torch.arange(n)[None, :] <= torch.arange(n)[:, None]     # [i, j]
    for h in range(hq):
        g = h // group
        s = (q[:, h, :] @ k[:, g, :].T) / math.sqrt(hd)
        s = torch.where(allowed, s, torch.full_like(s, -math.inf))
        e = torch.exp(s - s.max(dim=-1, keepdim=True).values)
        w = e / e.sum(dim=-1, keepdim=True)
        o[:, h, :] = w @ v[:, g, :]
    return o


def silu(z: torch.Tensor) -> torch.Tensor:
    return z / (1.0 + torch.exp(-z))


def forward_nodedup(cfg: Any, embed: Any, layers: Iterable[Mapping[str, Any]], gf: Any,
                    tok: Sequence[int], cu_seqlens: Sequence[int],
                    pos: Optional[Sequence[int]] = None,
                    sequences: Optional[Sequence[int]] = None,
                    dtype: torch.dtype = torch.float64) -> np.ndarray:
    """Final-norm hidden states of the requested sequences, concatenated in the order given.

    cfg needs the attributes n_layers, d, n_q_heads, n_kv_heads, head_dim, eps, rope_base,
    qk_norm.  ``embed`` is either the [vocab, d] table or a callable ids -> rows.  ``layers``
    yields one mapping per layer with g1, wq, wk, wv, gq, gk, wo, g2, wg, wu, wd, all in the
    logical [out, in] layout of y = W h.  ``sequences`` selects whole sequences (default: all).
    """
    tok = np.asarray(tok, dtype=np.int64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    B = len(cu) - 1
    seq_ids = list(range(B)) if sequences is None else [int(s) for s in sequences]
    hq, hkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim

    xs, ps = [], []
    for s in seq_ids:
        ids = tok[cu[s]:cu[s + 1]]
        rows = embed(ids) if callable(embed) else np.asarray(embed)[ids]
        xs.append(_t(rows, dtype))
        if pos is None:
            ps.append(torch.arange(len(ids), dtype=torch.int64))
        else:
            ps.append(torch.as_tensor(np.asarray(pos, dtype=np.int64)[cu[s]:cu[s + 1]]))

    n_layers = 0
    for lw in layers:
        n_layers += 1
        w = {k: _t(a, dtype) for k, a in lw.items()}
        for si in range(len(xs)):
            x, p = xs[si], ps[si]
            n = x.shape[0]
            if n == 0:
                continue
            a = rmsnorm(x, w["g1"], cfg.eps)
            q = (a @ w["wq"].T).reshape(n, hq, hd)
            k = (a @ w["wk"].T).reshape(n, hkv, hd)
            v = (a @ w["wv"].T).reshape(n, hkv, hd)
            if cfg.qk_norm:
                q = rmsnorm(q, w["gq"], cfg.eps)
                k = rmsnorm(k, w["gk"], cfg.eps)
            q = rope(q, p, cfg.rope_base)
            k = rope(k, p, cfg.rope_base)
            o = causal_attention(q, k, v).reshape(n, hq * hd)
            x = x + o @ w["wo"].T
            b = rmsnorm(x, w["g2"], cfg.eps)
            x = x + (silu(b @ w["wg"].T) * (b @ w["wu"].T)) @ w["wd"].T
            xs[si] = x
    assert n_layers == cfg.n_layers, "layer count does not match the config"
    gf_t = _t(gf, dtype)
    out = [rmsnorm(x, gf_t, cfg.eps) for x in xs]
    if not out:
        return np.zeros((0, cfg.d), dtype=np.float64)
    return torch.cat(out, dim=0).numpy()


def lm_head_logits(hidden: Any, w_lm: Any, rows: Any = None, dtype: torch.dtype = torch.float64) -> np.ndarray:
    """Algorithm 1, last block ("Output"): logits = LMHead(h), a bias-free linear map.

    hidden[n, d]: final-norm hidden states (what ``forward_nodedup`` returns); w_lm[vocab, d]: the
    head in [out, in] layout like every other matrix here (the embedding matrix itself when the head
    is tied); rows: optional indices into hidden (e.g. the last token of every sequence, or I_gather
    for logits in compact space).  Returns logits[len(rows) or n, vocab] = hidden[rows] @ w_lm^T.
    """
    h = _t(hidden, dtype)
    if rows is not None:
        h = h[torch.as_tensor(np.asarray(rows, dtype=np.int64))]
    return torch.matmul(h, _t(w_lm, dtype).T).numpy()
