"""GPU parity of radix_build_index against the index oracle: bit-exact maps."""
import numpy as np
import pytest
import torch

from oracle import radix_index as oracle_index
from paper_2601_15013_amd import binding, synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def test_toy_example():
    s, g, n = U.build_index_gpu([1, 2, 3, 1, 2, 4], [0, 3, 6])
    assert n == 4 and s.tolist() == [0, 1, 2, 0, 1, 3] and g.tolist() == [0, 1, 2, 5]


@pytest.mark.parametrize("pattern", synth.SHARING_PATTERNS)
def test_named_patterns(pattern):
    b = synth.sharing_pattern(pattern, 11)
    assert U.assert_index_parity(b.tok, b.cu_seqlens) == b.expected_n_compact


def test_empty_and_degenerate_inputs():
    s, g, n = U.build_index_gpu([], [0])                   # B = 0
    assert n == 0 and len(s) == 0
    s, g, n = U.build_index_gpu([], [0, 0, 0])             # only empty sequences
    assert n == 0
    U.assert_index_parity([5, 6, 5], [0, 0, 2, 2, 3])      # empty sequences in between
    U.assert_index_parity([7], [0, 1])                     # one token
    U.assert_index_parity([4, 5, 6, 4, 5, 4, 5, 6, 7], [0, 3, 5, 9])   # prefixes of one another
    U.assert_index_parity([1, 2, 3, 9, 2, 3], [0, 3, 6])   # path specificity: nothing merges
    # single sequence and no sharing: identity maps
    s, g, n = U.build_index_gpu(np.arange(1000) % 7, [0, 1000])
    assert n == 1000 and np.array_equal(s, np.arange(1000)) and np.array_equal(g, np.arange(1000))
    b = synth.no_sharing_batch(5, 32, 512, 1000)
    s, g, n = U.build_index_gpu(b.tok, b.cu_seqlens)
    assert n == b.N and np.array_equal(s, np.arange(b.N))
    # identical sequences 32 x 512
    tok = np.tile(np.arange(10, 522), 32)
    s, g, n = U.build_index_gpu(tok, np.arange(33) * 512)
    assert n == 512 and np.array_equal(s, np.tile(np.arange(512), 32)) and np.array_equal(g, np.arange(512))


def test_explicit_positions():
    U.assert_index_parity([1, 2, 1, 2], [0, 2, 4], [0, 1, 0, 1])
    n = U.assert_index_parity([1, 2, 1, 2], [0, 2, 4], [0, 1, 0, 5])
    assert n == 3


@pytest.mark.parametrize("seed", range(30))
def test_random_small_batches(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 40))
    vocab = int(rng.integers(1, 4))
    lens = rng.integers(0, 12, size=B)
    cu = np.concatenate([[0], np.cumsum(lens)])
    tok = rng.integers(0, vocab, size=int(cu[-1]))
    pos = None
    if seed % 3 == 0 and cu[-1]:
        pos = np.concatenate([np.arange(n) + int(rng.integers(0, 2)) for n in lens])
    U.assert_index_parity(tok, cu, pos)


@pytest.mark.parametrize("seed", range(6))
def test_random_deep_tries(seed):
    # many sequences, long shared runs that break at random depths (spans several 256-token
    # compare chunks and several rounds), tiny alphabet after the break
    rng = np.random.default_rng(100 + seed)
    B = int(rng.integers(50, 300))
    base = rng.integers(0, 50, size=1500)
    seqs = []
    for _ in range(B):
        n = int(rng.integers(1, 1500))
        s = base[:n].copy()
        for _ in range(int(rng.integers(0, 3))):
            cut = int(rng.integers(0, n))
            s[cut:] = rng.integers(0, 3, size=n - cut)
        seqs.append(s)
    cu = np.concatenate([[0], np.cumsum([len(s) for s in seqs])])
    U.assert_index_parity(np.concatenate(seqs), cu)


def test_large_batch_of_short_sequences():
    # B above one workgroup's thread count: the per-sequence loops stride
    rng = np.random.default_rng(7)
    B = 3000
    lens = rng.integers(0, 9, size=B)
    cu = np.concatenate([[0], np.cumsum(lens)])
    tok = rng.integers(0, 3, size=int(cu[-1]))
    U.assert_index_parity(tok, cu)


@pytest.mark.parametrize("key", ["C1", "C2", "C3", "C4", "C5", "C5ctl"])
def test_workloads_full_size(key):
    b = synth.make_batch(key)
    n = U.assert_index_parity(b.tok, b.cu_seqlens)
    assert n == b.expected_n_compact


def test_shuffled_multilevel():
    b = synth.multilevel_batch(9, 128, 256, 8, 32, 64, 192, 151936, shuffle=True)
    assert U.assert_index_parity(b.tok, b.cu_seqlens) == b.expected_n_compact


def test_device_data_errors_are_reported_not_faulted():
    dev = "cuda"
    tok = torch.tensor([1, 2, 3, 4], dtype=torch.int32, device=dev)
    ws = binding.alloc_workspace(binding.radix_index_workspace_bytes(2))
    for cu in ([0, 3, 2], [1, 2, 4], [0, 2, 5], [0, -1, 4]):
        cu_t = torch.tensor(cu, dtype=torch.int32, device=dev)
        with pytest.raises(binding.RadixError) as e:
            binding.radix_build_index(tok, None, cu_t, ws)
        assert e.value.code == -6
    bad_tok = torch.tensor([1, -2, 3, 4], dtype=torch.int32, device=dev)
    with pytest.raises(binding.RadixError) as e:
        binding.radix_build_index(bad_tok, None, torch.tensor([0, 2, 4], dtype=torch.int32, device=dev), ws)
    assert e.value.code == -7
    # the workspace is usable again afterwards
    I_s, I_g, _, n = binding.radix_build_index(tok, None, torch.tensor([0, 2, 4], dtype=torch.int32, device=dev), ws)
    assert n == 4 and binding.radix_device_status(ws) == 0


def test_async_call_then_status():
    dev = "cuda"
    b = synth.make_batch("C1")
    tok = torch.from_numpy(b.tok).to(dev); cu = torch.from_numpy(b.cu_seqlens).to(dev)
    ws = binding.alloc_workspace(binding.radix_index_workspace_bytes(b.B))
    I_s, I_g, n_dev, n = binding.radix_build_index(tok, None, cu, ws, sync=False)
    assert n is None
    assert binding.radix_device_status(ws) == 0
    assert int(n_dev.item()) == 160


def test_index_select_rows_matches_indexing():
    rng = np.random.default_rng(3)
    for shape, n_out, dt in [((100, 128), 200, torch.float32), ((1600, 1024), 7000, torch.bfloat16),
                             ((50, 3), 77, torch.float32), ((20, 64, 16), 100, torch.bfloat16)]:
        src = torch.from_numpy(rng.standard_normal(shape).astype(np.float32)).to(dt).cuda()
        idx = torch.from_numpy(rng.integers(0, shape[0], size=n_out).astype(np.int32)).cuda()
        out = binding.radix_index_select_rows(src, idx)
        assert torch.equal(out.cpu(), src.cpu()[idx.cpu().long()])
