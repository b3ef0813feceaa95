"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and rejects
host-visible argument errors before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

from paper_2601_15013_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2601_15013_amd import build
        build.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    inc = os.path.join(ROOT, "include")
    header = "\n".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    declared = set(re.findall(r"^(?:int|const char\*)\s+(radix_\w+)\s*\(", header, flags=re.M))
    assert declared == set(binding.EXPORTS)
    raw = C.CDLL(binding.LIB_PATH)
    for name in declared:
        assert getattr(raw, name) is not None


def test_status_strings(lib):
    assert binding.radix_status_string(0) == "ok"
    seen = {binding.radix_status_string(c) for c in range(-10, 1)}
    assert len(seen) == 11 and "unknown status" not in seen
    assert binding.radix_status_string(-99) == "unknown status"


def test_index_workspace_bytes(lib):
    a = binding.radix_index_workspace_bytes(0)
    b = binding.radix_index_workspace_bytes(256)
    c = binding.radix_index_workspace_bytes(4096)
    assert 256 < a <= b < c and b % 256 == 0
    with pytest.raises(binding.RadixError) as e:
        binding.radix_index_workspace_bytes(-1)
    assert e.value.code == -2


def test_build_index_rejects_bad_host_arguments(lib):
    i32 = C.c_int32
    fake = C.c_void_p(0x1000)          # never dereferenced: every call below fails its host checks
    host = i32(0)
    f = lib.radix_build_index
    assert f(fake, None, fake, -1, 4, fake, fake, fake, C.byref(host), fake, 1 << 20, None) == -2     # B < 0
    assert f(fake, None, fake, 2, -4, fake, fake, fake, C.byref(host), fake, 1 << 20, None) == -2     # N < 0
    assert f(fake, None, None, 2, 4, fake, fake, fake, C.byref(host), fake, 1 << 20, None) == -1      # cu NULL
    assert f(None, None, fake, 2, 4, fake, fake, fake, C.byref(host), fake, 1 << 20, None) == -1      # tok NULL
    assert f(fake, None, fake, 2, 4, fake, fake, fake, C.byref(host), None, 1 << 20, None) == -1      # ws NULL
    assert f(fake, None, fake, 0, 4, fake, fake, fake, C.byref(host), fake, 1 << 20, None) == -2      # tokens, no seqs
    assert f(fake, None, fake, 2, 4, fake, fake, fake, C.byref(host), C.c_void_p(0x1010), 1 << 20, None) == -5
    assert f(fake, None, fake, 2, 4, fake, fake, fake, C.byref(host), fake, 16, None) == -4           # ws too small


def test_forward_rejects_bad_host_arguments(lib):
    fake = C.c_void_p(0x1000)
    f = lib.radix_prefill_forward
    assert f(None, fake, None, fake, 1, 4, 4, fake, fake, 4, None, fake, fake, 1 << 20, None) == -1   # model NULL
    g = lib.radix_prefill_forward_nodedup
    assert g(None, fake, None, fake, 1, 4, 4, fake, fake, 1 << 20, None) == -1
    n = C.c_size_t()
    assert lib.radix_workspace_bytes(None, 4, 1, C.byref(n)) == -1
    assert lib.radix_model_hilo_layers(None) == -1


def test_model_create_rejects_bad_config(lib):
    out = C.c_void_p()
    assert lib.radix_model_create(None, None, C.byref(out)) == -1
    w = binding.radix_weights(0x1000, 0x1000, None, None)
    good = dict(n_layers=1, d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_int=768, vocab=10, max_pos=16,
                qk_norm=1, dtype=0, compute_dtype=0, hilo_layers=0, fold_norms=0, lm_head=0, eps=1e-6, rope_base=1e6)

    def create(**kw):
        c = binding.radix_model_config(**dict(good, **kw))
        return lib.radix_model_create(C.byref(c), C.byref(w), C.byref(out))

    assert create(n_kv_heads=3) == -9            # Hkv does not divide Hq
    assert create(n_layers=0) == -9
    assert create(head_dim=256) == -3            # head_dim > 128
    assert create(dtype=7) == -3
    assert create(dtype=1, compute_dtype=1) == -3    # 16-bit path needs head_dim 128
    assert create(compute_dtype=2) == -3         # fp32 weights are multiplied in fp32
    assert create(hilo_layers=1) == -3           # (hi, lo) activations exist for 16-bit operands only
    assert create(hilo_layers=-2) == -9
    assert create(hilo_layers=-1) == -1          # "none" is fine with fp32 weights (config passes, layers_host NULL)
    assert create(lm_head=3) == -9
    assert create(fold_norms=2) == -9
    assert create(dtype=1, compute_dtype=2, head_dim=128, n_q_heads=2, n_kv_heads=1, d=256, d_int=512, vocab=1000, lm_head=1) == -3   # 16-bit head: vocab % 128
    assert create(dtype=1, compute_dtype=0, head_dim=128) == -3
    assert create(d_int=100) == -3               # gate/up interleave needs multiples of 32
    assert create() == -1                        # config fine, layers_host NULL
    assert out.value is None


def test_lm_head_rejects_bad_host_arguments(lib):
    fake = C.c_void_p(0x1000)
    n = C.c_size_t()
    assert lib.radix_lm_head_workspace_bytes(None, 4, C.byref(n)) == -1
    assert lib.radix_lm_head(None, fake, 4, None, 4, fake, fake, 1 << 20, None) == -1      # model NULL


def test_index_select_rejects_bad_host_arguments(lib):
    fake = C.c_void_p(0x1000)
    f = lib.radix_index_select_rows
    assert f(fake, 4, fake, -1, 16, fake, None, None) == -2
    assert f(None, 4, fake, 2, 16, fake, None, None) == -1
    assert f(fake, 4, fake, 2, 6, fake, None, None) == -5      # row_bytes not a multiple of 4
    assert f(fake, 4, fake, 0, 16, fake, None, None) == 0      # nothing to do


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode == 2
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


def _header_struct_fields(name):
    """Field names of `typedef struct <name> { ... } <name>;` in include/radixmlp.h, in order."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(root, "include", "radixmlp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    body = re.search(r"typedef\s+struct\s+%s\s*\{(.*?)\}\s*%s\s*;" % (name, name), text, flags=re.S).group(1)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if decl:
            fields.append(re.findall(r"[A-Za-z_][A-Za-z_0-9]*", decl)[-1])
    return fields


@pytest.mark.parametrize("name", ["radix_model_config", "radix_layer_weights", "radix_weights", "radix_fwd_opts"])
def test_binding_structs_follow_the_header(name):
    # same fields in the same order: a field added to the header and not to the binding would shift every later one
    ctype = getattr(binding, name)
    assert [f[0] for f in ctype._fields_] == _header_struct_fields(name)
