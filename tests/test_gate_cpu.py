"""The gate that decides whether a batch is deduplicated (radix_dedup_decision: host arithmetic in the library, the
same function radix_prefill_forward calls), checked without a GPU.

Paper: Experiments (radix_mlp_threshold: deduplicate when the compact share is below the threshold; 0.0 turns
RadixMLP off) and Limitations, "Low-redundancy batches" (a batch that shares little is not worth the index
operations).  The automatic rule is this library's own cost model (documented at radix_fwd_opts.threshold); the tests
pin its structure - monotone in the number of rows saved, never deduplicates when nothing is shared, follows the
measured crossover of the paper's sweep shapes - not the exact constants."""
import os

import pytest

from paper_2601_15013_amd import binding, synth


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2601_15013_amd import build
        build.build()
    return binding.load_library()


def cfg_of(model_cfg, compute="f16"):
    return binding.make_config(model_cfg, compute_dtype=compute)


def sweep_counts(prefix, suffix, B=32):
    """N and N' of the paper's sweep batches (Appendix, compression ratio: one shared prefix + B distinct suffixes)."""
    return B * (prefix + suffix), prefix + B * suffix


def test_explicit_threshold_is_the_papers_rule(lib):
    c = cfg_of(synth.QWEN3_0_6B)
    N, n = 1000, 950
    assert binding.radix_dedup_decision(c, 8, N, n, threshold=1.0)
    assert binding.radix_dedup_decision(c, 8, N, n, threshold=0.96)
    assert not binding.radix_dedup_decision(c, 8, N, n, threshold=0.95)        # strict: 950 < 0.95 * 1000 is false
    assert not binding.radix_dedup_decision(c, 8, N, n, threshold=0.5)
    assert not binding.radix_dedup_decision(c, 8, N, n, threshold=0.0)         # the paper's "off"
    assert not binding.radix_dedup_decision(c, 8, N, N, threshold=1.0)         # nothing shared: N' < N is false
    assert binding.radix_dedup_decision(c, 8, N, N, threshold=0.0, force_dedup=True)


@pytest.mark.parametrize("fused", [None, False])
@pytest.mark.parametrize("model_cfg", [synth.QWEN3_0_6B, synth.QWEN3_4B, synth.QWEN3_8B])
def test_automatic_gate_structure(lib, model_cfg, fused):
    c = cfg_of(model_cfg)
    for suffix in (256, 1024):
        N, _ = sweep_counts(2048, suffix)
        # nothing shared: never
        assert not binding.radix_dedup_decision(c, 32, N, N, fused_attention=fused)
        # monotone: once a batch with n unique rows is deduplicated, every batch with fewer unique rows is
        decisions = [binding.radix_dedup_decision(c, 32, N, n, fused_attention=fused) for n in range(N, 0, -max(1, N // 200))]
        first = decisions.index(True)
        assert all(decisions[first:]), "not monotone in the rows saved"
        # a long shared prefix is always worth it
        assert binding.radix_dedup_decision(c, 32, *sweep_counts(2048, suffix), fused_attention=fused)
        assert binding.radix_dedup_decision(c, 32, *sweep_counts(512, suffix), fused_attention=fused)
        # one shared token is not on the small model (the index operations cost more than 31 rows save; on the
        # large shapes the two sides are within a few microseconds of each other and either answer is fine)
        if model_cfg is synth.QWEN3_0_6B:
            assert not binding.radix_dedup_decision(c, 32, *sweep_counts(1, suffix), fused_attention=fused)


def test_automatic_gate_weighs_the_model_size(lib):
    # The same batch: the larger the model, the more position-wise work a saved row is worth against the same
    # attention / copy overhead, so the break-even share N'/N moves up with the model.
    def break_even(model_cfg, fused):
        c = cfg_of(model_cfg)
        N = 32 * 1056
        n = N
        while n > 0 and not binding.radix_dedup_decision(c, 32, N, n, fused_attention=fused):
            n -= 16
        return n / N
    for fused in (None, False):
        small, mid, big = (break_even(m, fused) for m in (synth.QWEN3_0_6B, synth.QWEN3_4B, synth.QWEN3_8B))
        assert 0.5 < small <= mid <= big < 1.0, (fused, small, mid, big)


def test_gate_rejects_bad_arguments(lib):
    c = cfg_of(synth.QWEN3_0_6B)
    import ctypes as C
    out = C.c_int32(7)
    raw = lib
    assert raw.radix_dedup_decision(None, 1, 1, 1, None, C.byref(out)) == -1
    assert raw.radix_dedup_decision(C.byref(c), 1, 1, 1, None, None) == -1
    assert raw.radix_dedup_decision(C.byref(c), 1, 10, 11, None, C.byref(out)) == -2      # n_compact > N
    assert raw.radix_dedup_decision(C.byref(c), -1, 10, 5, None, C.byref(out)) == -2
    bad = binding.radix_fwd_opts(-1.0, 0, 9, 0)
    assert raw.radix_dedup_decision(C.byref(c), 1, 10, 5, C.byref(bad), C.byref(out)) < 0  # unknown attention mode
    f32 = cfg_of(synth.WORKLOADS["C1"].model, compute="f32")
    fused = binding.radix_fwd_opts(-1.0, 0, 2, 0)
    assert raw.radix_dedup_decision(C.byref(f32), 1, 10, 5, C.byref(fused), C.byref(out)) < 0   # fused needs 16-bit operands
    assert raw.radix_dedup_decision(C.byref(c), 4, 100, 50, None, C.byref(out)) == 0 and out.value in (0, 1)
