"""Pins for the index-map oracle (oracle/radix_index.py).  CPU only."""
import os

import numpy as np
import pytest

from oracle import radix_index as orc
from paper_2601_15013_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_kv(path):
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        out[k] = np.array([int(x) for x in v])
    return out


def check_invariants(tok, cu, scat, gath, pos=None):
    """Structural facts that hold for the unique valid answer at any size."""
    tok = np.asarray(tok); cu = np.asarray(cu)
    N = int(cu[-1]) if len(cu) else 0
    assert scat.shape == (N,)
    n_c = len(gath)
    if N == 0:
        assert n_c == 0
        return
    assert np.all(np.diff(gath) > 0), "I_gather strictly increasing"
    assert scat.max() + 1 == n_c
    assert np.array_equal(scat[gath], np.arange(n_c)), "I_scatter[I_gather[i]] == i"
    rep = gath[scat]
    assert np.all(rep <= np.arange(N)), "representative is the first occurrence"
    assert np.array_equal(tok[rep], tok), "representative carries the same token"
    p = orc._positions(cu, pos)
    assert np.array_equal(p[rep], p), "... and the same position"
    first = True
    for s in range(len(cu) - 1):
        seg = scat[cu[s]:cu[s + 1]]
        if len(seg) == 0:
            continue
        assert np.all(np.diff(seg) > 0), "a child node is created after its parent"
        if first:
            assert np.array_equal(seg, np.arange(len(seg))), "first sequence is all new nodes"
            first = False


@pytest.mark.parametrize("fn", [orc.build_index_trie, orc.build_index_bruteforce])
def test_toy_example(fn):
    g = _read_kv(os.path.join(GOLDEN, "toy_example.txt"))
    scat, gath = fn(g["tok"], g["cu_seqlens"])
    assert scat.tolist() == g["I_scatter"].tolist()
    assert gath.tolist() == g["I_gather"].tolist()
    assert scat.dtype == np.int32 and gath.dtype == np.int32
    # "4 unique nodes from 6 tokens": gamma = N'/N = 4/6
    r, gamma = orc.compression(6, len(gath))
    assert abs(gamma - 0.667) < 1e-3 and abs(r - 1.5) < 1e-12


def test_closed_form_table_rows():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "prefix_suffix_counts.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 15
    for P, S, N, Np in [[int(x) for x in r] for r in rows]:
        assert N == 32 * (P + S) and Np == P + 32 * S          # the closed form itself
        if N > 20000:
            continue                                           # keep the CPU suite short
        b = synth.shared_prefix_batch(7, 32, P, S, S, 50000)
        assert b.N == N
        scat, gath = orc.build_index_trie(b.tok, b.cu_seqlens)
        assert len(gath) == Np
        check_invariants(b.tok, b.cu_seqlens, scat, gath)
        # the paper's worked ratios: r = 7.2 for 2048/256 (too large here) and
        # gamma column of the table, e.g. 0.515 for 256/256
    r, gamma = orc.compression(32 * 2304, 2048 + 32 * 256)
    assert abs(r - 7.2) < 1e-12
    r, _ = orc.compression(32 * 3072, 2048 + 32 * 1024)
    assert abs(r - 2.8235) < 1e-3


def test_c1_counts():
    b = synth.make_batch("C1")
    assert (b.B, b.N) == (8, 384)
    scat, gath = orc.build_index_trie(b.tok, b.cu_seqlens)
    assert len(gath) == 160 == b.expected_n_compact
    check_invariants(b.tok, b.cu_seqlens, scat, gath)
    s2, g2 = orc.build_index_bruteforce(b.tok, b.cu_seqlens)
    assert np.array_equal(s2, scat) and np.array_equal(g2, gath)


def test_trivial_cases_are_identity():
    # single sequence, and no sharing: identity maps
    b = synth.sharing_pattern("single_sequence", 3)
    scat, gath = orc.build_index_trie(b.tok, b.cu_seqlens)
    assert scat.tolist() == list(range(5)) == gath.tolist()
    b = synth.no_sharing_batch(5, 32, 64, 1000)
    scat, gath = orc.build_index_trie(b.tok, b.cu_seqlens)
    assert np.array_equal(scat, np.arange(b.N)) and np.array_equal(gath, np.arange(b.N))
    # identical sequences: B copies of 0..L-1
    seq = np.arange(10, 522)
    tok = np.tile(seq, 32); cu = np.arange(33) * 512
    scat, gath = orc.build_index_trie(tok, cu)
    assert np.array_equal(scat, np.tile(np.arange(512), 32))
    assert np.array_equal(gath, np.arange(512))


def test_empty_inputs():
    for fn in (orc.build_index_trie, orc.build_index_bruteforce):
        scat, gath = fn([], [0])
        assert len(scat) == 0 and len(gath) == 0
        scat, gath = fn([], [0, 0, 0])
        assert len(scat) == 0 and len(gath) == 0
        scat, gath = fn([5, 6, 5], [0, 0, 2, 2, 3])     # empty sequences in between
        assert scat.tolist() == [0, 1, 0] and gath.tolist() == [0, 1]


def test_path_specificity():
    # Same (token, position) after different prefixes must not merge (Problem Formulation).
    tok = [1, 2, 3, 9, 2, 3]
    scat, gath = orc.build_index_trie(tok, [0, 3, 6])
    assert scat.tolist() == [0, 1, 2, 3, 4, 5]
    # re-converging is impossible: after one differing token everything below is new
    tok = [1, 2, 3, 4, 1, 7, 3, 4]
    scat, gath = orc.build_index_trie(tok, [0, 4, 8])
    assert scat.tolist() == [0, 1, 2, 3, 0, 4, 5, 6] and gath.tolist() == [0, 1, 2, 3, 5, 6, 7]


def test_explicit_positions_enter_the_key():
    tok = [1, 2, 1, 2]
    s, g = orc.build_index_trie(tok, [0, 2, 4], pos=[0, 1, 0, 1])
    assert s.tolist() == [0, 1, 0, 1]
    s, g = orc.build_index_trie(tok, [0, 2, 4], pos=[0, 1, 0, 5])   # same tokens, other position
    assert s.tolist() == [0, 1, 0, 2] and g.tolist() == [0, 1, 3]
    assert orc.node_key(3, 7) == (3 << 32) + 7
    assert orc.node_key(1, 5) != orc.node_key(5, 1)


def test_prefix_of_another_sequence_and_order():
    # a sequence that is a strict prefix of an earlier one adds no node; a later, longer one
    # only adds its tail; numbering is creation order
    tok = [4, 5, 6, 4, 5, 4, 5, 6, 7]
    scat, gath = orc.build_index_trie(tok, [0, 3, 5, 9])
    assert scat.tolist() == [0, 1, 2, 0, 1, 0, 1, 2, 3]
    assert gath.tolist() == [0, 1, 2, 8]


@pytest.mark.parametrize("seed", range(40))
def test_trie_matches_definition_on_random_batches(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 7))
    vocab = int(rng.integers(1, 4))              # tiny vocab => lots of accidental sharing
    lens = rng.integers(0, 7, size=B)
    cu = np.concatenate([[0], np.cumsum(lens)])
    tok = rng.integers(0, vocab, size=int(cu[-1]))
    pos = None
    if seed % 3 == 0:                            # explicit, sometimes clashing, positions
        pos = np.concatenate([np.arange(n) + int(rng.integers(0, 2)) for n in lens]) if cu[-1] else []
    a = orc.build_index_trie(tok, cu, pos)
    b = orc.build_index_bruteforce(tok, cu, pos)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    check_invariants(tok, cu, a[0], a[1], pos)


@pytest.mark.parametrize("pattern", synth.SHARING_PATTERNS)
def test_named_sharing_patterns(pattern):
    b = synth.sharing_pattern(pattern, 11)
    want_tokens = {"single_sequence": 5, "identical_sequences": 10, "shared_prefix": 10,
                   "no_sharing": 6, "mixed_lengths": 10, "complex_sharing": 20}[pattern]
    assert b.N == want_tokens                    # token counts of the paper's validation table
    a = orc.build_index_trie(b.tok, b.cu_seqlens)
    d = orc.build_index_bruteforce(b.tok, b.cu_seqlens)
    assert np.array_equal(a[0], d[0]) and np.array_equal(a[1], d[1])
    assert len(a[1]) == b.expected_n_compact
    check_invariants(b.tok, b.cu_seqlens, a[0], a[1])


@pytest.mark.parametrize("key", ["C2", "C3"])
def test_workload_counts_follow_closed_form(key):
    b = synth.make_batch(key)
    scat, gath = orc.build_index_trie(b.tok, b.cu_seqlens)
    assert len(gath) == b.expected_n_compact
    check_invariants(b.tok, b.cu_seqlens, scat, gath)


def test_shuffled_multilevel_batch():
    b = synth.multilevel_batch(9, 16, 12, 4, 5, 3, 9, 500, shuffle=True)
    scat, gath = orc.build_index_trie(b.tok, b.cu_seqlens)
    assert len(gath) == b.expected_n_compact
    d = orc.build_index_bruteforce(b.tok, b.cu_seqlens)
    assert np.array_equal(scat, d[0]) and np.array_equal(gath, d[1])
