"""The fused attention mode (scatter and gather folded into the attention kernel, representative
positions only) against the three-kernel path and the fp64 no-dedup oracle.

The fused kernel walks the same K/V tiles in the same order and every row's arithmetic is that of
the full-layout kernel, so the two modes must agree bit for bit; the oracle bound is the one of
tests/test_gpu_forward.py.
"""
import numpy as np
import pytest
import torch

from paper_2601_15013_amd import binding, harness, synth
from tests import gpu_util as U
from tests.test_gpu_forward import SMALL_BF16, TOL_BF16

pytestmark = pytest.mark.gpu


def run_modes(weights, batch, pos=None):
    model = harness.upload_model(weights)
    try:
        run = harness.Runner(model, batch.N, batch.B)
        tok, cu = harness.upload_batch(batch)
        pos_t = None if pos is None else torch.from_numpy(np.asarray(pos, dtype=np.int32)).cuda()
        maps = run.build_index(tok, cu, pos_t)
        y = run.forward(tok, cu, batch.max_seqlen, maps, pos=pos_t, force_dedup=True,
                        fused_attention=False).cpu().numpy()
        assert run.status() == 0
        y_f = run.forward(tok, cu, batch.max_seqlen, maps, pos=pos_t, force_dedup=True,
                          fused_attention=True).cpu().numpy()
        assert run.status() == 0
        return y, y_f, maps[3]
    finally:
        model.close()


@pytest.mark.parametrize("pattern", synth.SHARING_PATTERNS)
def test_fused_equals_three_kernel_path_on_sharing_patterns(pattern):
    w = synth.SynthWeights(SMALL_BF16, 41)
    b = synth.sharing_pattern(pattern, 12)
    y, y_f, _ = run_modes(w, b)
    assert np.array_equal(y, y_f)
    assert U.rel_err(y_f, U.oracle_rows(w, b)) <= TOL_BF16


def test_fused_ragged_multilevel_several_tiles_explicit_positions():
    # sequences span several K/V tiles, representative suffixes start at arbitrary offsets
    w = synth.SynthWeights(SMALL_BF16, 42)
    b = synth.multilevel_batch(6, 12, 150, 3, 40, 1, 300, SMALL_BF16.vocab)
    pos = np.concatenate([np.arange(n) + 5 for n in np.diff(b.cu_seqlens)])
    y, y_f, n_c = run_modes(w, b, pos=pos)
    assert n_c == b.expected_n_compact
    assert np.array_equal(y, y_f)
    assert U.rel_err(y_f, U.oracle_rows(w, b, pos=pos)) <= TOL_BF16


@pytest.mark.parametrize("heads", [(4, 2), (2, 2), (8, 2)])
def test_fused_short_suffixes_of_different_sequences_share_a_workgroup(heads):
    # Suffixes of at most 32 representative rows behind long shared prefixes: with 2 (or 4) row slots per workgroup
    # the leftover blocks of consecutive sequences are packed together and walk the common prefix's K/V tiles
    # once.  (4, 2): two slots; (2, 2): four slots, one head per workgroup; (8, 2): one slot, nothing to pack.
    hq, hkv = heads
    cfg = synth.ModelConfig("bf16p", 2, 256, hq, hkv, 128, 320, 2000, "bf16", max_pos=1024)
    w = synth.SynthWeights(cfg, 45)
    # three-level trie: 200 shared, 4 groups x 70, then suffixes of 1..40 tokens (some sequences one block, some two,
    # first query positions not tile-aligned); and a flat one with empty and one-token suffixes
    deep = synth.multilevel_batch(10, 24, 200, 4, 70, 1, 40, cfg.vocab)
    flat = synth.shared_prefix_batch(11, 13, 333, 0, 32, cfg.vocab)
    mixed = synth.multilevel_batch(12, 10, 130, 5, 3, 20, 110, cfg.vocab)      # 1 to 4 blocks per sequence
    for b in (deep, flat, mixed):
        y, y_f, n_c = run_modes(w, b)
        assert n_c == b.expected_n_compact
        assert np.array_equal(y, y_f), b.name
        assert U.rel_err(y_f, U.oracle_rows(w, b)) <= TOL_BF16


def test_fused_whole_sequences_duplicated_and_tiny_batches():
    w = synth.SynthWeights(SMALL_BF16, 43)
    one = synth.shared_prefix_batch(1, 1, 0, 70, 70, SMALL_BF16.vocab)
    tok = np.concatenate([one.tok, one.tok, one.tok[:30], one.tok]).astype(np.int32)        # copies and a prefix
    cu = np.array([0, 70, 140, 170, 240], dtype=np.int32)
    dup = synth.Batch("copies", tok, cu, 70)
    for b in (dup, synth.shared_prefix_batch(2, 1, 0, 1, 1, 2000), synth.shared_prefix_batch(3, 3, 1, 1, 3, 2000)):
        y, y_f, n_c = run_modes(w, b)
        assert n_c == b.expected_n_compact
        assert np.array_equal(y, y_f)
        assert U.rel_err(y_f, U.oracle_rows(w, b)) <= TOL_BF16


def test_fused_mode_needs_16bit_operands_and_follows_the_threshold():
    # fp32 configuration: refused
    w32 = synth.make_weights("C1")
    b = synth.make_batch("C1")
    model = harness.upload_model(w32)
    run = harness.Runner(model, b.N, b.B)
    tok, cu = harness.upload_batch(b)
    maps = run.build_index(tok, cu)
    with pytest.raises(binding.RadixError) as e:
        run.forward(tok, cu, b.max_seqlen, maps, fused_attention=True)
    assert e.value.code == -3
    model.close()
    # deduplication gated off by the threshold: the flag is ignored, result = no-dedup pass
    w = synth.SynthWeights(SMALL_BF16, 44)
    b = synth.shared_prefix_batch(4, 6, 20, 30, 60, SMALL_BF16.vocab)
    model = harness.upload_model(w)
    run = harness.Runner(model, b.N, b.B)
    tok, cu = harness.upload_batch(b)
    maps = run.build_index(tok, cu)
    y_off = run.forward(tok, cu, b.max_seqlen, maps, threshold=0.0, fused_attention=True).cpu().numpy()
    y_nd = run.forward_nodedup(tok, cu, b.max_seqlen).cpu().numpy()
    assert run.status() == 0
    assert np.array_equal(y_off, y_nd)
    model.close()


def _full_size(key, sequences):
    b = synth.make_batch(key)
    w = synth.make_weights(key)
    y, y_f, n_c = run_modes(w, b)
    assert n_c == b.expected_n_compact
    assert np.array_equal(y, y_f)           # every row of the full batch
    if sequences:
        rows = U.rows_of(b, sequences)
        err = U.rel_err(y_f[rows], U.oracle_rows(w, b, sequences=sequences))
        print(f"{key} fused: sampled rows={len(rows)} err={err:.3e}")
        assert err <= TOL_BF16


def test_fused_c2_full_size():
    _full_size("C2", [0, 33, 63])


def test_fused_c3_full_size_three_level_trie():
    _full_size("C3", [])


def test_fused_c5_full_size_long_shared_prefix():
    _full_size("C5", [127])
