"""LM head (Algorithm 1, output block) on the GPU against the fp64 oracle: logits of selected rows,
tied and separate heads, and the compact-space order of Algorithm 1 (head on N' rows, then scatter)."""
import dataclasses
import numpy as np
import pytest
import torch

from oracle import forward as oracle_forward
from paper_2601_15013_amd import binding, harness, synth
from tests import gpu_util as U
from tests.test_gpu_forward import SMALL_BF16, TOL_BF16, TOL_F32

pytestmark = pytest.mark.gpu


def _forward(model, batch):
    run = harness.Runner(model, batch.N, batch.B)
    tok, cu = harness.upload_batch(batch)
    maps = run.build_index(tok, cu)
    y = run.forward(tok, cu, batch.max_seqlen, maps)
    assert run.status() == 0
    return run, maps, y


def test_fp32_tied_head_last_token_logits():
    b = synth.make_batch("C1")
    w = synth.make_weights("C1")
    model = harness.upload_model(w, lm_head_mode=1)
    run, maps, y = _forward(model, b)
    last = (b.cu_seqlens[1:] - 1).astype(np.int32)
    ws = binding.alloc_workspace(binding.radix_lm_head_workspace_bytes(model, len(last)))
    logits = binding.radix_lm_head(model, y, torch.from_numpy(last).cuda(), ws).cpu().numpy()
    assert binding.radix_device_status(ws) == 0
    ref = oracle_forward.lm_head_logits(U.oracle_rows(w, b), w.embed, rows=last)
    assert logits.shape == ref.shape == (b.B, w.cfg.vocab)
    assert U.rel_err(logits, ref) <= TOL_F32
    # all rows, no selection list
    ws_all = binding.alloc_workspace(binding.radix_lm_head_workspace_bytes(model, b.N))
    all_logits = binding.radix_lm_head(model, y, None, ws_all).cpu().numpy()
    assert np.array_equal(all_logits[last], logits)
    model.close()


@pytest.mark.parametrize("head", [1, 2])
def test_bf16_head_tied_and_separate_compact_space_then_scatter(head):
    cfg = dataclasses.replace(SMALL_BF16, vocab=2048)
    w = synth.SynthWeights(cfg, 51)
    lm = None
    if head == 2:
        rng = np.random.Generator(np.random.Philox(key=[51, 0x4EAD]))
        lm = synth._round_to_bf16((0.02 * rng.standard_normal((cfg.vocab, cfg.d))).astype(np.float32))
    b = synth.multilevel_batch(7, 10, 40, 2, 20, 1, 90, cfg.vocab)
    model = harness.upload_model(w, lm_head=lm, lm_head_mode=head)
    run, maps, y = _forward(model, b)
    I_s, I_g, _, n_c = maps
    w_head = w.embed if head == 1 else lm
    ref_hidden = U.oracle_rows(w, b)
    # last token of every sequence (what a reranker reads)
    last = (b.cu_seqlens[1:] - 1).astype(np.int32)
    ws = binding.alloc_workspace(binding.radix_lm_head_workspace_bytes(model, b.N))
    logits = binding.radix_lm_head(model, y, torch.from_numpy(last).cuda(), ws).cpu().numpy()
    ref = oracle_forward.lm_head_logits(ref_hidden, w_head, rows=last)
    err = U.rel_err(logits, ref)
    print(f"lm head ({'tied' if head == 1 else 'separate'}): last-token logits err {err:.3e}")
    assert err <= TOL_BF16
    # Algorithm 1's order: logits in compact space, then scatter; equals the head on all N rows bit for bit
    y_c = binding.radix_lm_head(model, y, I_g[:n_c].contiguous(), ws)
    y_scattered = binding.radix_index_select_rows(y_c, I_s).cpu().numpy()
    y_all = binding.radix_lm_head(model, y, None, ws).cpu().numpy()
    assert binding.radix_device_status(ws) == 0
    assert np.array_equal(y_scattered, y_all)
    assert U.rel_err(y_all, oracle_forward.lm_head_logits(ref_hidden, w_head)) <= TOL_BF16
    model.close()


def test_lm_head_errors_and_empty_selection():
    cfg = dataclasses.replace(SMALL_BF16, vocab=2048)
    w = synth.SynthWeights(cfg, 52)
    model = harness.upload_model(w, lm_head_mode=1)
    hidden = torch.zeros((5, cfg.d), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(binding.radix_lm_head_workspace_bytes(model, 8))
    out = binding.radix_lm_head(model, hidden, torch.zeros(0, dtype=torch.int32, device="cuda"), ws)
    assert out.shape == (0, cfg.vocab)
    # a row index outside the hidden states: clamped, reported, nothing faults
    bad = torch.tensor([0, 7, -1], dtype=torch.int32, device="cuda")
    out = binding.radix_lm_head(model, hidden, bad, ws)
    torch.cuda.synchronize()
    assert binding.radix_device_status(ws) == -7
    assert torch.all(out == 0)
    with pytest.raises(binding.RadixError) as e:        # workspace too small
        binding.radix_lm_head(model, hidden, None, binding.alloc_workspace(256))
    assert e.value.code == -4
    model.close()
    # a model created without a head refuses
    model = harness.upload_model(synth.SynthWeights(cfg, 52))
    with pytest.raises(binding.RadixError) as e:
        binding.radix_lm_head(model, hidden, None, ws)
    assert e.value.code == -3
    model.close()


def test_c2_shape_last_token_logits():
    # full vocabulary (151 936 = 1187 x 128 columns), head tied to the embedding, B = 64 selected rows
    b = synth.make_batch("C2")
    w = synth.make_weights("C2")
    model = harness.upload_model(w, lm_head_mode=1)
    run, maps, y = _forward(model, b)
    last = (b.cu_seqlens[1:] - 1).astype(np.int32)
    ws = binding.alloc_workspace(binding.radix_lm_head_workspace_bytes(model, b.B))
    logits = binding.radix_lm_head(model, y, torch.from_numpy(last).cuda(), ws).cpu().numpy()
    assert binding.radix_device_status(ws) == 0
    seqs = [0, 63]
    ref_hidden = U.oracle_rows(w, b, sequences=seqs)
    ends = np.cumsum([b.cu_seqlens[s + 1] - b.cu_seqlens[s] for s in seqs]) - 1
    ref = oracle_forward.lm_head_logits(ref_hidden, w.embed, rows=ends)
    err = U.rel_err(logits[seqs], ref)
    print(f"C2 last-token logits over the full vocabulary: err {err:.3e}")
    assert err <= TOL_BF16
    model.close()
