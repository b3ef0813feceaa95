"""Shared helpers of the GPU parity tests."""
import numpy as np
import torch

from oracle import forward as oracle_forward
from oracle import radix_index as oracle_index
from paper_2601_15013_amd import binding, harness, synth


def have_gpu() -> bool:
    return torch.cuda.is_available()


def build_index_gpu(tok_np, cu_np, pos_np=None):
    """Run radix_build_index on numpy inputs; returns (I_scatter, I_gather[:N'], N') as numpy."""
    dev = "cuda"
    tok = torch.from_numpy(np.asarray(tok_np, dtype=np.int32)).to(dev)
    cu = torch.from_numpy(np.asarray(cu_np, dtype=np.int32)).to(dev)
    pos = None if pos_np is None else torch.from_numpy(np.asarray(pos_np, dtype=np.int32)).to(dev)
    ws = binding.alloc_workspace(binding.radix_index_workspace_bytes(len(cu_np) - 1))
    I_s, I_g, n_dev, n = binding.radix_build_index(tok, pos, cu, ws)
    assert int(n_dev.item()) == n
    return I_s.cpu().numpy(), I_g[:n].cpu().numpy(), n


def assert_index_parity(tok_np, cu_np, pos_np=None):
    s_ref, g_ref = oracle_index.build_index_trie(tok_np, cu_np, pos_np)
    s, g, n = build_index_gpu(tok_np, cu_np, pos_np)
    assert n == len(g_ref)
    assert np.array_equal(g, g_ref), "I_gather differs from the oracle"
    assert np.array_equal(s, s_ref), "I_scatter differs from the oracle"
    return n


def oracle_rows(weights, batch, sequences=None, pos=None):
    cfg = weights.cfg
    return oracle_forward.forward_nodedup(cfg, weights.embed, weights.layers, weights.gf, batch.tok,
                                          batch.cu_seqlens, pos=pos, sequences=sequences)


def rows_of(batch, sequences):
    cu = batch.cu_seqlens
    return np.concatenate([np.arange(cu[s], cu[s + 1]) for s in sequences]) if len(sequences) else np.zeros(0, int)


def rel_err(y, ref):
    """max |err| relative to the RMS of the oracle's output."""
    rms = float(np.sqrt(np.mean(np.asarray(ref, dtype=np.float64) ** 2)))
    return float(np.max(np.abs(np.asarray(y, dtype=np.float64) - ref))) / rms


def rms_err(y, ref):
    """RMS of the error relative to the RMS of the oracle's output."""
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.sqrt(np.mean((np.asarray(y, dtype=np.float64) - ref) ** 2)) / np.sqrt(np.mean(ref ** 2)))


def tail_factor(n_sampled: int, n_all: int) -> float:
    """How much further out the largest of n_all error entries sits than the largest of n_sampled, for errors with a
    Gaussian tail: the expected maximum of n draws of |N(0, s)| grows like s * sqrt(2 ln(2 n)).  A maximum measured on
    a sample of the outputs is multiplied by this before it is compared with a tolerance that is meant for all of them."""
    if n_sampled >= n_all:
        return 1.0
    return float(np.sqrt(np.log(2.0 * n_all) / np.log(2.0 * n_sampled)))
