"""Seeded synthetic inputs: model shapes, random-init weights and ragged token batches.

This module only *makes inputs*.  It holds none of the method's arithmetic (no trie, no
index maps, no forward pass): the CPU oracle and the HIP library both receive the plain
arrays produced here and neither imports this module.

Randomness is counter-based (numpy's Philox bit generator keyed by
``(seed, tensor id, chunk)``), so any tensor can be regenerated on demand without holding
a whole multi-billion-parameter model in host memory.

Workload shapes follow the paper's two workload families (Experiments, synthetic
prefix/suffix batches; reranking batches with a shared template+query prefix and
per-candidate passage suffixes of roughly 75-200 tokens).  The paper's own data set,
tokenizer and trained weights are not used: token ids are uniform random and weights are
N(0, 0.02) draws.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_CHUNK = 1 << 24  # elements per independently keyed chunk of a tensor


@dataclasses.dataclass(frozen=True)
class ModelConfig:
    """Shape of a Qwen3-style causal decoder."""

    name: str
    n_layers: int
    d: int            # hidden size
    n_q_heads: int    # Hq
    n_kv_heads: int   # Hkv
    head_dim: int     # hd
    d_int: int        # SwiGLU intermediate size
    vocab: int
    dtype: str        # "f32" or "bf16": type the weights are generated, rounded and handed over in
    eps: float = 1e-6
    rope_base: float = 1e6
    qk_norm: bool = True
    max_pos: int = 4096

    @property
    def dq(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def dkv(self) -> int:
        return self.n_kv_heads * self.head_dim


TINY = ModelConfig("tiny", 2, 256, 4, 2, 64, 768, 1024, "f32", max_pos=512)
QWEN3_0_6B = ModelConfig("qwen3-0.6b", 28, 1024, 16, 8, 128, 3072, 151936, "bf16")
QWEN3_4B = ModelConfig("qwen3-4b", 36, 2560, 32, 8, 128, 9728, 151936, "bf16")
QWEN3_8B = ModelConfig("qwen3-8b", 36, 4096, 32, 8, 128, 12288, 151936, "bf16")


def _round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).copy()
    t = u >> np.uint32(16)
    t &= np.uint32(1)
    t += np.uint32(0x7FFF)
    u += t                      # wraps like the 32-bit hardware add; finite inputs never reach the wrap
    u &= np.uint32(0xFFFF0000)
    return u.view(np.float32)


def _normal_chunk(seed: int, tid: int, chunk: int, n: int) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=[(seed << 20) ^ tid, chunk]))
    return rng.standard_normal(n, dtype=np.float32)


_POOL: Optional[ThreadPoolExecutor] = None


def _pool() -> ThreadPoolExecutor:
    global _POOL
    if _POOL is None:
        _POOL = ThreadPoolExecutor(max(1, min(16, os.cpu_count() or 8)))
    return _POOL


def _chunk_jobs(seed: int, tid: int, out: np.ndarray, std: float, mean: float, bf16: bool):
    """One job per independently keyed chunk of a flat fp32 array: draw, scale, shift, round - all in place."""
    n = out.size
    jobs = []
    for c, lo in enumerate(range(0, n, _CHUNK)):
        hi = min(n, lo + _CHUNK)

        def run(c=c, lo=lo, hi=hi):
            x = _normal_chunk(seed, tid, c, hi - lo)
            x *= np.float32(std)
            if mean != 0.0:
                x += np.float32(mean)
            out[lo:hi] = _round_to_bf16(x) if bf16 else x
        jobs.append(run)
    return jobs


def _run_jobs(jobs) -> None:
    if len(jobs) > 1:
        list(_pool().map(lambda j: j(), jobs))
    else:
        for j in jobs:
            j()


def seeded_normal(seed: int, tid: int, shape: Tuple[int, ...], std: float, mean: float = 0.0,
                  bf16: bool = False) -> np.ndarray:
    """fp32 array of N(mean, std) draws, a pure function of (seed, tid, shape)."""
    out = np.empty(int(np.prod(shape)), dtype=np.float32)
    _run_jobs(_chunk_jobs(seed, tid, out, std, mean, bf16))
    return out.reshape(shape)


_LAYER_TENSORS = ("g1", "wq", "wk", "wv", "gq", "gk", "wo", "g2", "wg", "wu", "wd")


class SynthWeights:
    """Random-init weights of a ModelConfig, generated lazily and deterministically.

    Matrices and the embedding are N(0, 0.02); RMSNorm gains are 1 + N(0, 0.02) so that the
    gain multiply stays visible to tests without collapsing activations.  All matrices use
    the logical ``[out, in]`` row-major layout of ``y = W h``.  For bf16 configs every value
    is rounded to bf16 (nearest even) and handed out as fp32.
    """

    def __init__(self, cfg: ModelConfig, seed: int):
        self.cfg = cfg
        self.seed = int(seed)
        self._bf16 = cfg.dtype == "bf16"

    def _shape(self, name: str) -> Tuple[int, ...]:
        c = self.cfg
        return {
            "embed": (c.vocab, c.d), "gf": (c.d,),
            "g1": (c.d,), "g2": (c.d,), "gq": (c.head_dim,), "gk": (c.head_dim,),
            "wq": (c.dq, c.d), "wk": (c.dkv, c.d), "wv": (c.dkv, c.d), "wo": (c.d, c.dq),
            "wg": (c.d_int, c.d), "wu": (c.d_int, c.d), "wd": (c.d, c.d_int),
        }[name]

    @staticmethod
    def _tid(name: str, layer: int) -> int:
        if name in ("embed", "gf"):
            return 1 if name == "embed" else 2
        return 16 + layer * 16 + _LAYER_TENSORS.index(name)

    def tensor(self, name: str, layer: int = -1) -> np.ndarray:
        return seeded_normal(self.seed, self._tid(name, layer), self._shape(name), 0.02,
                             mean=1.0 if name.startswith("g") else 0.0, bf16=self._bf16)

    def layer(self, l: int) -> Dict[str, np.ndarray]:
        """All tensors of layer l; the chunks of all of them are drawn side by side."""
        flat = {n: np.empty(int(np.prod(self._shape(n))), dtype=np.float32) for n in _LAYER_TENSORS}
        jobs = []
        for n in _LAYER_TENSORS:
            jobs += _chunk_jobs(self.seed, self._tid(n, l), flat[n], 0.02, 1.0 if n.startswith("g") else 0.0, self._bf16)
        _run_jobs(jobs)
        return {n: flat[n].reshape(self._shape(n)) for n in _LAYER_TENSORS}

    # sequence-of-layers view (lazy): ``weights.layers[l]["wq"]``
    @property
    def layers(self) -> "_LazyLayers":
        return _LazyLayers(self)

    @property
    def embed(self) -> np.ndarray:
        return self.tensor("embed")

    def embed_rows(self, ids: np.ndarray) -> np.ndarray:
        """Embedding rows for the given token ids (generates the table once)."""
        return self.tensor("embed")[ids]

    @property
    def gf(self) -> np.ndarray:
        return self.tensor("gf")


class _LazyLayers:
    def __init__(self, w: SynthWeights):
        self._w = w

    def __len__(self) -> int:
        return self._w.cfg.n_layers

    def __getitem__(self, l: int) -> Dict[str, np.ndarray]:
        if not 0 <= l < len(self):
            raise IndexError(l)
        return self._w.layer(l)

    def __iter__(self):
        for l in range(len(self)):
            yield self[l]


# --------------------------------------------------------------------------------------
# Ragged token batches
# --------------------------------------------------------------------------------------

@dataclasses.dataclass
class Batch:
    name: str
    tok: np.ndarray          # int32 [N]
    cu_seqlens: np.ndarray   # int32 [B+1]
    expected_n_compact: Optional[int] = None  # closed-form N' when the recipe fixes it

    @property
    def B(self) -> int:
        return len(self.cu_seqlens) - 1

    @property
    def N(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def max_seqlen(self) -> int:
        return int(np.diff(self.cu_seqlens).max()) if self.B else 0


def _tokens(rng: np.random.Generator, n: int, vocab: int) -> np.ndarray:
    return rng.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def _distinct_first(rng: np.random.Generator, suffixes: List[np.ndarray], vocab: int) -> None:
    """Re-draw so that sibling suffixes differ in their first token.

    Makes the trie size equal the closed form P + sum(S_i): no accidental sharing between
    "distinct" branches.
    """
    seen = set()
    for s in suffixes:
        if len(s) == 0:
            continue
        while int(s[0]) in seen:
            s[0] = rng.integers(0, vocab)
        seen.add(int(s[0]))


def _assemble(name: str, seqs: Sequence[np.ndarray], n_compact: Optional[int]) -> Batch:
    lens = np.array([len(s) for s in seqs], dtype=np.int64)
    cu = np.zeros(len(seqs) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    tok = np.concatenate(seqs).astype(np.int32) if len(seqs) else np.zeros(0, np.int32)
    return Batch(name, tok, cu, n_compact)


def shared_prefix_batch(seed: int, B: int, prefix: int, suffix_lo: int, suffix_hi: int,
                        vocab: int, name: str = "shared_prefix") -> Batch:
    """B sequences = one shared prefix + a distinct suffix with length uniform in [lo, hi]."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0xBA7C]))
    lens = rng.integers(suffix_lo, suffix_hi + 1, size=B)
    pre = _tokens(rng, prefix, vocab)
    suf = [_tokens(rng, int(n), vocab) for n in lens]
    _distinct_first(rng, suf, vocab)
    seqs = [np.concatenate([pre, s]) for s in suf]
    return _assemble(name, seqs, prefix + int(lens.sum()))


def multilevel_batch(seed: int, B: int, prefix: int, n_groups: int, group_len: int,
                     suffix_lo: int, suffix_hi: int, vocab: int, shuffle: bool = False,
                     name: str = "multilevel") -> Batch:
    """Shared prefix, then one of n_groups distinct query blocks, then a unique suffix.

    Sequence s uses query block ``s // (B // n_groups)`` (contiguous groups) unless
    ``shuffle`` permutes the sequence order.
    """
    assert B % n_groups == 0
    rng = np.random.Generator(np.random.Philox(key=[seed, 0xBA7C]))
    lens = rng.integers(suffix_lo, suffix_hi + 1, size=B)
    pre = _tokens(rng, prefix, vocab)
    groups = [_tokens(rng, group_len, vocab) for _ in range(n_groups)]
    _distinct_first(rng, groups, vocab)
    per = B // n_groups
    suf = [_tokens(rng, int(n), vocab) for n in lens]
    for g in range(n_groups):
        _distinct_first(rng, suf[g * per:(g + 1) * per], vocab)
    seqs = [np.concatenate([pre, groups[s // per], suf[s]]) for s in range(B)]
    if shuffle:
        order = rng.permutation(B)
        seqs = [seqs[i] for i in order]
    n_compact = prefix + n_groups * group_len + int(lens.sum())
    return _assemble(name, seqs, n_compact)


def no_sharing_batch(seed: int, B: int, length: int, vocab: int, name: str = "no_sharing") -> Batch:
    """B sequences of the same length whose first tokens are all distinct (N' = N)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0xBA7C]))
    seqs = [_tokens(rng, length, vocab) for _ in range(B)]
    _distinct_first(rng, seqs, vocab)
    return _assemble(name, seqs, B * length)


def sharing_pattern(pattern: str, seed: int, vocab: int = 1024) -> Batch:
    """Small batches named after the paper's six prefix-sharing validation patterns
    (Appendix "Training Validation"): names and token counts follow the paper's table,
    contents are our own seeded draws."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x9A77]))
    t = lambda n: _tokens(rng, n, vocab)
    if pattern == "single_sequence":      # 5 tokens
        return _assemble(pattern, [t(5)], 5)
    if pattern == "identical_sequences":  # 2 x 5 = 10 tokens
        s = t(5)
        return _assemble(pattern, [s.copy(), s.copy()], 5)
    if pattern == "shared_prefix":        # 10 tokens: prefix 3 + suffixes 2 and 2
        p = t(3)
        suf = [t(2), t(2)]
        _distinct_first(rng, suf, vocab)
        return _assemble(pattern, [np.concatenate([p, s]) for s in suf], 3 + 4)
    if pattern == "no_sharing":           # 6 tokens
        suf = [t(3), t(3)]
        _distinct_first(rng, suf, vocab)
        return _assemble(pattern, suf, 6)
    if pattern == "mixed_lengths":        # 10 tokens: lengths 2, 3, 5 sharing a 2-token prefix
        p = t(2)
        suf = [t(0), t(1), t(3)]
        _distinct_first(rng, suf, vocab)
        return _assemble(pattern, [np.concatenate([p, s]) for s in suf], 2 + 1 + 3)
    if pattern == "complex_sharing":      # 20 tokens, branching at several depths
        a, b, c = t(3), t(2), t(2)
        x = [t(1), t(2)]
        _distinct_first(rng, x, vocab)
        y = [b, t(3)]
        _distinct_first(rng, y, vocab)
        seqs = [np.concatenate([a, y[0], x[0]]),      # 6
                np.concatenate([a, y[0], x[1]]),      # 7
                np.concatenate([a, y[1]]),            # 6
                c[:1]]                                # 1
        # the 4th sequence must not start like the others
        while int(seqs[3][0]) == int(a[0]):
            seqs[3][0] = rng.integers(0, vocab)
        assert sum(len(s) for s in seqs) == 20
        return _assemble(pattern, seqs, 3 + 2 + 1 + 2 + 3 + 1)
    raise ValueError(pattern)


SHARING_PATTERNS = ("single_sequence", "identical_sequences", "shared_prefix", "no_sharing",
                    "mixed_lengths", "complex_sharing")


# --------------------------------------------------------------------------------------
# The five named configurations (model shape + batch recipe + seed)
# --------------------------------------------------------------------------------------

@dataclasses.dataclass(frozen=True)
class Workload:
    key: str
    model: ModelConfig
    seed: int
    description: str


WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", TINY, 1001, "tiny fp32: 8 x (32 shared + 16 own)"),
    "C2": Workload("C2", QWEN3_0_6B, 1002, "0.6B bf16 rerank: 64 x (48 shared + U[64,192])"),
    "C3": Workload("C3", QWEN3_4B, 1003, "4B bf16 multilevel: 128 x (256 + 8 groups x 32 + U[64,192])"),
    "C4": Workload("C4", QWEN3_8B, 1004, "8B bf16 rerank: 256 x (64 shared + U[96,256])"),
    "C5": Workload("C5", QWEN3_0_6B, 1005, "0.6B bf16 long prefix: 128 x (2048 shared + 32 own)"),
    "C5ctl": Workload("C5ctl", QWEN3_0_6B, 1006, "0.6B bf16 control: 128 x 2080, no sharing"),
}


def make_batch(key: str) -> Batch:
    w = WORKLOADS[key]
    v = w.model.vocab
    if key == "C1":
        return shared_prefix_batch(w.seed, 8, 32, 16, 16, v, name=key)
    if key == "C2":
        return shared_prefix_batch(w.seed, 64, 48, 64, 192, v, name=key)
    if key == "C3":
        return multilevel_batch(w.seed, 128, 256, 8, 32, 64, 192, v, name=key)
    if key == "C4":
        return shared_prefix_batch(w.seed, 256, 64, 96, 256, v, name=key)
    if key == "C5":
        return shared_prefix_batch(w.seed, 128, 2048, 32, 32, v, name=key)
    if key == "C5ctl":
        return no_sharing_batch(w.seed, 128, 2080, v, name=key)
    raise KeyError(key)


def make_weights(key: str) -> SynthWeights:
    w = WORKLOADS[key]
    return SynthWeights(w.model, w.seed)
