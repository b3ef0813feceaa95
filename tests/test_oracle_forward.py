"""Pins for the forward oracle (oracle/forward.py).  CPU only.

The paper prints no activation values, so the oracle is pinned by (i) a second
composition made only of torch's own library routines, (ii) closed forms and
(iii) invariants the method relies on (causality, batch independence, duplicates).
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import forward as orc
from paper_2601_15013_amd import synth

SMALL = synth.ModelConfig("small", 2, 32, 4, 2, 8, 48, 97, "f32", max_pos=64)


def _weights(cfg, seed=5):
    w = synth.SynthWeights(cfg, seed)
    return w.embed, [w.layer(l) for l in range(cfg.n_layers)], w.gf


def library_forward(cfg, embed, layers, gf, tok, cu, pos=None):
    """Same model, written only with torch library routines, float64."""
    f = lambda a: torch.as_tensor(np.asarray(a)).double()
    outs = []
    for s in range(len(cu) - 1):
        ids = torch.as_tensor(np.asarray(tok[cu[s]:cu[s + 1]], dtype=np.int64))
        n = len(ids)
        if n == 0:
            continue
        p = torch.arange(n).double() if pos is None else f(pos[cu[s]:cu[s + 1]])
        x = F.embedding(ids, f(embed))
        hd = cfg.head_dim
        inv = 1.0 / (cfg.rope_base ** (torch.arange(0, hd, 2).double() / hd))
        rot = torch.polar(torch.ones(n, hd // 2).double(), p[:, None] * inv[None, :])   # e^{i p theta}

        def rope(t):      # complex rotation of the pair (t_i, t_{i+hd/2})
            z = torch.complex(t[..., :hd // 2], t[..., hd // 2:]) * rot[:, None, :]
            return torch.cat([z.real, z.imag], dim=-1)

        for w in layers:
            a = F.rms_norm(x, (cfg.d,), f(w["g1"]), cfg.eps)
            q = F.linear(a, f(w["wq"])).view(n, cfg.n_q_heads, hd)
            k = F.linear(a, f(w["wk"])).view(n, cfg.n_kv_heads, hd)
            v = F.linear(a, f(w["wv"])).view(n, cfg.n_kv_heads, hd)
            if cfg.qk_norm:
                q = F.rms_norm(q, (hd,), f(w["gq"]), cfg.eps)
                k = F.rms_norm(k, (hd,), f(w["gk"]), cfg.eps)
            q, k = rope(q), rope(k)
            rep = cfg.n_q_heads // cfg.n_kv_heads
            kk = k.repeat_interleave(rep, dim=1)
            vv = v.repeat_interleave(rep, dim=1)
            o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kk.transpose(0, 1)[None],
                                               vv.transpose(0, 1)[None], is_causal=True)[0]
            o = o.transpose(0, 1).reshape(n, cfg.dq)
            x = x + F.linear(o, f(w["wo"]))
            b = F.rms_norm(x, (cfg.d,), f(w["g2"]), cfg.eps)
            x = x + F.linear(F.silu(F.linear(b, f(w["wg"]))) * F.linear(b, f(w["wu"])), f(w["wd"]))
        outs.append(F.rms_norm(x, (cfg.d,), f(gf), cfg.eps))
    return torch.cat(outs).numpy() if outs else np.zeros((0, cfg.d))


def _run(cfg, wts, tok, cu, **kw):
    return orc.forward_nodedup(cfg, wts[0], wts[1], wts[2], tok, cu, **kw)


def test_matches_library_composition_small():
    wts = _weights(SMALL)
    rng = np.random.default_rng(0)
    lens = [5, 1, 9, 0, 3]
    cu = np.concatenate([[0], np.cumsum(lens)])
    tok = rng.integers(0, SMALL.vocab, size=cu[-1])
    y = _run(SMALL, wts, tok, cu)
    z = library_forward(SMALL, *wts, tok, cu)
    assert y.shape == (cu[-1], SMALL.d)
    assert np.max(np.abs(y - z)) < 1e-12


def test_matches_library_composition_explicit_positions_and_no_qknorm():
    cfg = synth.ModelConfig("small2", 1, 32, 4, 4, 8, 40, 50, "f32", qk_norm=False, rope_base=100.0)
    wts = _weights(cfg, 8)
    tok = np.arange(12) % 50
    cu = np.array([0, 7, 12])
    pos = np.array([3, 4, 5, 6, 7, 8, 9, 0, 2, 4, 6, 8])
    y = _run(cfg, wts, tok, cu, pos=pos)
    z = library_forward(cfg, *wts, tok, cu, pos=pos)
    assert np.max(np.abs(y - z)) < 1e-12


def test_matches_library_composition_c1():
    cfg = synth.TINY
    b = synth.make_batch("C1")
    w = synth.make_weights("C1")
    wts = (w.embed, [w.layer(l) for l in range(cfg.n_layers)], w.gf)
    y = _run(cfg, wts, b.tok, b.cu_seqlens)
    z = library_forward(cfg, *wts, b.tok, b.cu_seqlens)
    rms = math.sqrt(np.mean(z * z))
    assert 0.5 < rms < 2.0
    assert np.max(np.abs(y - z)) / rms < 1e-12


def test_weight_layout_is_out_by_in():
    # y = W h with W[out, in]: explicit scalar loops on one projection
    cfg = SMALL
    emb, layers, gf = _weights(cfg)
    a = np.linspace(-1, 1, cfg.d)
    w = np.asarray(layers[0]["wq"], dtype=np.float64)
    want = [sum(w[o, i] * a[i] for i in range(cfg.d)) for o in range(cfg.dq)]
    got = (torch.as_tensor(a)[None] @ torch.as_tensor(w).T)[0].numpy()
    assert np.allclose(got, want, atol=1e-14)
    assert w.shape == (cfg.dq, cfg.d) and np.asarray(layers[0]["wd"]).shape == (cfg.d, cfg.d_int)


def test_rmsnorm_closed_forms():
    x = torch.tensor([[3.0, -4.0]], dtype=torch.float64)
    g = torch.tensor([2.0, 0.5], dtype=torch.float64)
    # mean square = 12.5
    y = orc.rmsnorm(x, g, 0.0)
    assert torch.allclose(y, torch.tensor([[6.0 / math.sqrt(12.5), -2.0 / math.sqrt(12.5)]], dtype=torch.float64))
    # eps sits inside the square root
    y = orc.rmsnorm(torch.zeros(1, 4, dtype=torch.float64) + 1e-3, torch.ones(4, dtype=torch.float64), 1e-6)
    assert torch.allclose(y, torch.full((1, 4), 1e-3 / math.sqrt(2e-6), dtype=torch.float64))


def test_rope_properties():
    hd = 8
    rng = np.random.default_rng(1)
    q = torch.as_tensor(rng.standard_normal((6, 1, hd)))
    k = torch.as_tensor(rng.standard_normal((6, 1, hd)))
    p = torch.arange(6)
    rq, rk = orc.rope(q, p, 1e4), orc.rope(k, p, 1e4)
    assert torch.allclose(rq[0], q[0])                               # position 0: identity
    assert torch.allclose(rq.norm(dim=-1), q.norm(dim=-1))           # rotation keeps the norm
    # relative-position property: <R_m q, R_n k> depends on m - n only
    q0, k0 = q[0, 0], k[0, 0]
    qq = orc.rope(q0.expand(6, 1, hd).clone(), p, 1e4)
    kk = orc.rope(k0.expand(6, 1, hd).clone(), p, 1e4)
    assert torch.allclose((qq[3, 0] * kk[1, 0]).sum(), (qq[5, 0] * kk[3, 0]).sum())
    assert not torch.allclose((qq[3, 0] * kk[1, 0]).sum(), (qq[3, 0] * kk[2, 0]).sum())
    # first pair (i = 0, theta = 1) at position 1 is a rotation by one radian of (x_0, x_{hd/2})
    x = torch.zeros(2, 1, hd, dtype=torch.float64); x[:, 0, 0] = 1.0
    r = orc.rope(x, torch.tensor([0, 1]), 1e4)
    assert abs(r[1, 0, 0] - math.cos(1.0)) < 1e-15 and abs(r[1, 0, hd // 2] - math.sin(1.0)) < 1e-15
    # last pair rotates by base^(-(hd-2)/hd)
    x = torch.zeros(2, 1, hd, dtype=torch.float64); x[:, 0, hd // 2 - 1] = 1.0
    r = orc.rope(x, torch.tensor([0, 2]), 1e4)
    th = 1e4 ** (-(hd - 2) / hd)
    assert abs(r[1, 0, hd // 2 - 1] - math.cos(2 * th)) < 1e-15 and abs(r[1, 0, hd - 1] - math.sin(2 * th)) < 1e-15


def test_attention_closed_forms():
    rng = np.random.default_rng(2)
    n, hq, hkv, hd = 5, 4, 2, 8
    q = torch.as_tensor(rng.standard_normal((n, hq, hd)))
    k = torch.as_tensor(rng.standard_normal((n, hkv, hd)))
    v = torch.as_tensor(rng.standard_normal((n, hkv, hd)))
    o = orc.causal_attention(q, k, v)
    # the first query only sees the first key: output is v_0 of its KV group
    for h in range(hq):
        assert torch.allclose(o[0, h], v[0, h // 2])
    # zero queries give uniform weights: running mean of v
    o = orc.causal_attention(torch.zeros_like(q), k, v)
    for i in range(n):
        assert torch.allclose(o[i, 3], v[: i + 1, 1].mean(dim=0))
    # one dominant key: weight exp(s)/(exp(s)+i) on it
    q1 = torch.zeros(n, hq, hd, dtype=torch.float64); q1[:, :, 0] = math.sqrt(hd)
    k1 = torch.zeros(n, hkv, hd, dtype=torch.float64); k1[0, :, 0] = 2.0
    o = orc.causal_attention(q1, k1, v)
    wgt = math.exp(2.0) / (math.exp(2.0) + 3)
    assert torch.allclose(o[3, 0], wgt * v[0, 0] + (1 - wgt) / 3 * v[1:4, 0].sum(dim=0))


def test_zero_output_projections_reduce_to_norm_of_embedding():
    cfg = SMALL
    emb, layers, gf = _weights(cfg)
    layers = [dict(l, wo=np.zeros_like(l["wo"]), wd=np.zeros_like(l["wd"])) for l in layers]
    tok = np.array([3, 1, 4, 1, 5]); cu = np.array([0, 5])
    y = _run(cfg, (emb, layers, gf), tok, cu)
    e = np.asarray(emb, dtype=np.float64)[tok]
    want = e / np.sqrt((e * e).mean(axis=1, keepdims=True) + cfg.eps) * np.asarray(gf, dtype=np.float64)
    assert np.max(np.abs(y - want)) < 1e-13


def test_single_token_sequence_closed_form():
    # one token: attention output = v, so the layer is a chain of position-wise maps
    cfg = synth.ModelConfig("one", 1, 16, 2, 1, 8, 24, 11, "f32")
    emb, layers, gf = _weights(cfg, 3)
    w = {k: np.asarray(a, dtype=np.float64) for k, a in layers[0].items()}
    tok = np.array([7]); cu = np.array([0, 1])
    y = _run(cfg, (emb, layers, gf), tok, cu)[0]
    norm = lambda x, g: x / math.sqrt(float(np.mean(x * x)) + cfg.eps) * g
    x = np.asarray(emb, dtype=np.float64)[7]
    v = w["wv"] @ norm(x, w["g1"])
    x = x + w["wo"] @ np.concatenate([v, v])          # both query heads read KV head 0
    b = norm(x, w["g2"])
    gate = w["wg"] @ b
    x = x + w["wd"] @ (gate / (1 + np.exp(-gate)) * (w["wu"] @ b))
    assert np.max(np.abs(y - norm(x, np.asarray(gf, dtype=np.float64)))) < 1e-13


def test_causality_batch_independence_and_duplicates():
    cfg = SMALL
    wts = _weights(cfg)
    rng = np.random.default_rng(4)
    a = rng.integers(0, cfg.vocab, size=9)
    b = rng.integers(0, cfg.vocab, size=6)
    y_a = _run(cfg, wts, a, [0, 9])
    # causality: truncating a sequence leaves the earlier rows unchanged
    y_trunc = _run(cfg, wts, a[:5], [0, 5])
    assert np.max(np.abs(y_a[:5] - y_trunc)) < 1e-13
    # ... and changing a later token does not change earlier rows, but changes later ones
    a2 = a.copy(); a2[6] = (a2[6] + 1) % cfg.vocab
    y_a2 = _run(cfg, wts, a2, [0, 9])
    assert np.max(np.abs(y_a2[:6] - y_a[:6])) == 0.0 and np.max(np.abs(y_a2[6:] - y_a[6:])) > 1e-3
    # batch independence and duplicates: [a, b, a] gives a's rows twice and b's own rows
    tok = np.concatenate([a, b, a]); cu = [0, 9, 15, 24]
    y = _run(cfg, wts, tok, cu)
    assert np.array_equal(y[:9], y_a) and np.array_equal(y[15:], y_a)
    assert np.array_equal(y[9:15], _run(cfg, wts, b, [0, 6]))
    # sequence subset selection returns whole sequences in the order asked
    ysub = _run(cfg, wts, tok, cu, sequences=[1, 0])
    assert np.array_equal(ysub[:6], y[9:15]) and np.array_equal(ysub[6:], y[:9])


def test_shared_prefix_rows_agree_across_sequences():
    # the property the method rests on: tokens with identical causal history have identical rows
    cfg = synth.TINY
    b = synth.make_batch("C1")
    w = synth.make_weights("C1")
    y = orc.forward_nodedup(cfg, w.embed, w.layers, w.gf, b.tok, b.cu_seqlens, sequences=[0, 5])
    assert np.array_equal(y[:32], y[48:80])
    assert not np.allclose(y[32:48], y[80:96])


def test_float32_mode_is_close_to_float64():
    cfg = SMALL
    wts = _weights(cfg)
    tok = np.arange(10) % cfg.vocab
    y64 = _run(cfg, wts, tok, [0, 10])
    y32 = _run(cfg, wts, tok, [0, 10], dtype=torch.float32)
    assert np.max(np.abs(y64 - y32)) < 1e-4


def test_lm_head_is_the_plain_linear_map():
    # pinned by the definition written as explicit sums, by unit vectors (a one-hot hidden state reads out
    # a column of the head) and by row selection commuting with the product
    rng = np.random.default_rng(7)
    hidden = rng.standard_normal((5, 6))
    w = rng.standard_normal((9, 6))
    got = orc.lm_head_logits(hidden, w)
    want = np.zeros((5, 9))
    for i in range(5):
        for v in range(9):
            for k in range(6):
                want[i, v] += hidden[i, k] * w[v, k]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    eye = np.eye(6)
    np.testing.assert_array_equal(orc.lm_head_logits(eye, w), w.T)
    rows = [4, 0, 0, 2]
    np.testing.assert_array_equal(orc.lm_head_logits(hidden, w, rows=rows), got[rows])
    assert orc.lm_head_logits(hidden, w, rows=[]).shape == (0, 9)


def test_lm_head_in_compact_space_then_scatter_equals_head_on_all_rows():
    # Algorithm 1's tail: y_c = LMHead(h_c), y = Scatter(y_c).  With the maps of a shared-prefix batch and
    # hidden states that are equal on duplicate rows (which the forward guarantees), both orders agree exactly.
    from oracle import radix_index as oracle_index
    b = synth.shared_prefix_batch(5, 4, 6, 2, 5, 50)
    I_s, I_g = oracle_index.build_index_trie(b.tok, b.cu_seqlens)
    rng = np.random.default_rng(8)
    h_c = rng.standard_normal((len(I_g), 7))
    h = h_c[I_s]                                  # rows of duplicates are copies
    w = rng.standard_normal((11, 7))
    y_c = orc.lm_head_logits(h, w, rows=I_g)
    np.testing.assert_array_equal(y_c[I_s], orc.lm_head_logits(h, w))
