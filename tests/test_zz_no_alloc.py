"""radix_build_index_static (the entry point that allocates nothing: builder state in the library's static
device array) against radix_build_index (caller-provided workspace): identical maps, bit for bit, on two calls
in a row, the second with a smaller input, so that state left by the first call cannot leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2601_15013_amd import binding, synth

pytestmark = pytest.mark.gpu


def _both(batch):
    tok = torch.from_numpy(batch.tok.astype(np.int32)).cuda()
    cu = torch.from_numpy(batch.cu_seqlens.astype(np.int32)).cuda()
    N = tok.numel()
    ws = binding.alloc_workspace(binding.radix_index_workspace_bytes(batch.B))
    s_ref, g_ref, _, n_ref = binding.radix_build_index(tok, None, cu, ws)
    # every buffer of the static call is allocated before it; poisoned so that unwritten entries show
    s = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    g = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    n_dev = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    n = binding.radix_build_index_static(tok, None, cu, s, g, n_dev)
    assert torch.cuda.memory_allocated() == before
    assert n == n_ref == int(n_dev.item())
    assert torch.equal(s, s_ref), "I_scatter differs from radix_build_index"
    assert torch.equal(g[:n], g_ref[:n]), "I_gather differs from radix_build_index"
    return n


def test_static_scratch_index_builder_matches_workspace_builder_twice():
    big = synth.multilevel_batch(41, 384, 60, 8, 12, 1, 90, 5000)        # 384 sequences, three trie levels, ragged
    small = synth.shared_prefix_batch(42, 7, 9, 1, 30, 5000)             # then a much smaller batch
    n_big = _both(big)
    n_small = _both(small)
    assert n_big == big.expected_n_compact and n_small == small.expected_n_compact
    # not synchronising (the form a graph capture would use): N' only on the device
    tok = torch.from_numpy(small.tok.astype(np.int32)).cuda()
    cu = torch.from_numpy(small.cu_seqlens.astype(np.int32)).cuda()
    s = torch.empty(tok.numel(), dtype=torch.int32, device="cuda")
    g = torch.empty(tok.numel(), dtype=torch.int32, device="cuda")
    n_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert binding.radix_build_index_static(tok, None, cu, s, g, n_dev, sync=False) is None
    assert int(n_dev.item()) == n_small


def test_static_scratch_index_builder_limits_and_errors():
    lib = binding.load_library()
    fake = C.c_void_p(0x1000)                  # never dereferenced: rejected on the host
    host = C.c_int32(0)
    too_many = 4096 + 1
    assert lib.radix_build_index_static(fake, None, fake, too_many, 4, fake, fake, fake, C.byref(host), None) == -10
    assert "static" in binding.radix_status_string(-10)
    assert lib.radix_build_index_static(fake, None, None, 2, 4, fake, fake, fake, C.byref(host), None) == -1
    # malformed cu_seqlens (device data): reported through the synchronising form, N' = 0
    tok = torch.tensor([1, 2, 3, 4], dtype=torch.int32, device="cuda")
    cu = torch.tensor([0, 3, 2], dtype=torch.int32, device="cuda")
    s = torch.full((4,), -7, dtype=torch.int32, device="cuda")
    g = torch.full((4,), -7, dtype=torch.int32, device="cuda")
    n_dev = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.RadixError) as e:
        binding.radix_build_index_static(tok, None, cu, s, g, n_dev)
    assert e.value.code == -6 and int(n_dev.item()) == 0
    # and the next well-formed call is unaffected
    cu = torch.tensor([0, 2, 4], dtype=torch.int32, device="cuda")
    assert binding.radix_build_index_static(tok, None, cu, s, g, n_dev) == 4
