"""The C-ABI library: loads without a GPU, exports every symbol include/ddtree.h declares, and
rejects bad arguments on the host before anything is launched (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ddtree.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2604_12989_amd.build import LIB, build_library
    if not os.path.exists(LIB):
        build_library()
    import paper_2604_12989_amd as dd
    return dd.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ddtree_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"ddtree_topk", "ddtree_build", "ddtree_verify_attn", "ddtree_accept",
            "ddtree_compact", "ddtree_workspace_bytes", "ddtree_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_covers_every_entry_point(lib):
    from paper_2604_12989_amd import binding
    assert set(declared_functions()) == set(binding._SIGNATURES)


def test_version_and_error_strings(lib):
    import paper_2604_12989_amd as dd
    assert dd.version() >= 100
    assert dd.error_string(0) == "ok"
    for code in (-1, -2, -3):
        assert dd.error_string(code) not in ("ok", "unknown error code")
    assert dd.error_string(-99) == "unknown error code"


def test_workspace_sizing_is_host_arithmetic(lib):
    import paper_2604_12989_amd as dd
    assert dd.workspace_bytes(1, 8, 1024, 16, 2, 1, 64, 128) >= 256
    big = dd.workspace_bytes(1, 16, 151936, 256, 32, 8, 128, 8192)
    assert 8e6 < big < 40e6            # dominated by the fp16 split-KV partials of the attention
    assert dd.workspace_bytes(1, 16, 151936, 256, 32, 7, 128, 8192) == 0   # Hq % Hkv != 0
    assert dd.workspace_bytes(1, 16, 151936, 4096, 32, 8, 128, 8192) == 0  # N above the maximum
    assert dd.workspace_bytes(0, 16, 151936, 256, 32, 8, 128, 8192) == 0


def test_attention_launch_arithmetic_selfcheck(lib):
    """The decomposition of the attention into workgroups, decoded on the host the way the kernel
    decodes it (reciprocal divisions, per-XCD runs, key ranges): every (sequence, KV head, row
    tile, key range) exactly once, rows and key tiles partitioned, equal to plain division."""
    import paper_2604_12989_amd as dd
    assert dd.selftest_host() == 0


def test_attention_scratch_never_exceeds_the_workspace_bound(lib):
    # ddtree_workspace_bytes must cover ddtree_verify_attn for every cache length: sweep budgets,
    # head layouts and lengths (the split of the key range, hence the scratch, depends on all three)
    import ctypes
    lib.ddtree_verify_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.ddtree_verify_attn_workspace_bytes.argtypes = [ctypes.c_int] * 6 + [ctypes.c_longlong]
    worst = 0.0
    for batch, Hq, Hkv in ((1, 32, 8), (1, 8, 2), (1, 4, 4), (2, 16, 2), (4, 32, 8), (16, 64, 8), (1, 64, 8)):
        for N in (1, 7, 8, 15, 16, 31, 32, 63, 64, 65, 100, 127, 128, 200, 255, 256, 257, 300, 511, 512, 1024):
            bound = lib.ddtree_workspace_bytes(batch, 16, 151936, N, Hq, Hkv, 128, 1 << 30)
            assert bound > 0
            for L in (0, 1, 63, 64, 65, 200, 257, 1000, 2048, 4097, 8192, 20000, 32768, 100000, 1 << 20):
                need = lib.ddtree_verify_attn_workspace_bytes(batch, N + 1, Hq, Hkv, 128, 0, batch * L)
                assert need <= bound, (batch, Hq, Hkv, N, L, need, bound)
                worst = max(worst, need / bound)
    assert worst > 0.2   # the bound is not vacuous


def test_bad_arguments_are_rejected_before_any_launch(lib):
    ERR_ARG, ERR_WS = -1, -2
    buf = ctypes.create_string_buffer(4096)
    p = ctypes.cast(buf, ctypes.c_void_p)
    # null pointers
    assert lib.ddtree_topk(None, 1, 1, 8, 1, p, p, p, 4096, None) == ERR_ARG
    # K > V, B out of range
    assert lib.ddtree_topk(p, 1, 1, 8, 9, p, p, p, 4096, None) == ERR_ARG
    assert lib.ddtree_topk(p, 1, 64, 8, 2, p, p, p, 4096, None) == ERR_ARG
    # workspace missing / too small
    assert lib.ddtree_topk(p, 1, 16, 151936, 256, p, p, None, 0, None) == ERR_WS
    assert lib.ddtree_topk(p, 1, 16, 151936, 256, p, p, p, 4096, None) == ERR_WS
    # build: N out of range
    assert lib.ddtree_build(p, p, 1, 8, 16, 0, p, p, p, p, p, p, p, p, None, 0, None) == ERR_ARG
    assert lib.ddtree_build(p, p, 1, 8, 16, 5000, p, p, p, p, p, p, p, p, None, 0, None) == ERR_ARG
    # attention: Hq not a multiple of Hkv, bad dtype, bad scale, decreasing kv_offset
    off = (ctypes.c_int32 * 2)(0, 128)
    offp = ctypes.cast(off, ctypes.c_void_p)
    assert lib.ddtree_verify_attn(p, p, p, p, p, p, offp, 1, 17, 3, 2, 64, 0.125, 1, p, None, 0, None) == ERR_ARG
    assert lib.ddtree_verify_attn(p, p, p, p, p, p, offp, 1, 17, 2, 1, 64, 0.125, 7, p, None, 0, None) == ERR_ARG
    assert lib.ddtree_verify_attn(p, p, p, p, p, p, offp, 1, 17, 2, 1, 64, -1.0, 1, p, None, 0, None) == ERR_ARG
    bad = (ctypes.c_int32 * 2)(5, 3)
    assert lib.ddtree_verify_attn(p, p, p, p, p, p, ctypes.cast(bad, ctypes.c_void_p), 1, 17, 2, 1, 64,
                                  0.125, 1, p, None, 0, None) == ERR_ARG
    # bf16 D=128 needs its split-KV scratch
    off2 = (ctypes.c_int32 * 2)(0, 8192)
    assert lib.ddtree_verify_attn(p, p, p, p, p, p, ctypes.cast(off2, ctypes.c_void_p), 1, 257, 32, 8,
                                  128, 0.088, 0, p, None, 0, None) == ERR_WS
    # tensors of the attention are read 16 bytes at a time: a misaligned one is refused
    odd = ctypes.c_void_p(p.value + 2)
    assert lib.ddtree_verify_attn(odd, p, p, p, p, p, ctypes.cast(off2, ctypes.c_void_p), 1, 257, 32, 8,
                                  128, 0.088, 0, p, None, 0, None) == ERR_ARG
    assert lib.ddtree_verify_attn(p, p, p, p, odd, p, ctypes.cast(off2, ctypes.c_void_p), 1, 257, 32, 8,
                                  128, 0.088, 0, p, None, 0, None) == ERR_ARG
    # spans of the cache: negative start or length
    st_ = (ctypes.c_int32 * 1)(-1)
    ln_ = (ctypes.c_int32 * 1)(5)
    assert lib.ddtree_verify_attn_spans(p, p, p, p, p, p, ctypes.cast(st_, ctypes.c_void_p),
                                        ctypes.cast(ln_, ctypes.c_void_p), 1, 17, 2, 1, 64, ctypes.c_float(0.125), 1, p,
                                        None, 0, None) == ERR_ARG
    assert lib.ddtree_verify_attn_spans(p, p, p, p, p, p, ctypes.cast(ln_, ctypes.c_void_p),
                                        ctypes.cast(st_, ctypes.c_void_p), 1, 17, 2, 1, 64, ctypes.c_float(0.125), 1, p,
                                        None, 0, None) == ERR_ARG
    # accept: workspace too small, null outputs
    assert lib.ddtree_accept(p, 1, 257, 151936, p, p, p, p, p, p, p, None, 16, p, 16, None) == ERR_WS
    assert lib.ddtree_accept(p, 1, 257, 151936, p, p, p, p, None, p, p, None, 16, p, 4096, None) == ERR_ARG
    # the variant with its scratch in the library's static array: null output, and a shape whose
    # partials exceed the array (64 sequences of 1025 rows), refused before any GPU call
    assert lib.ddtree_accept_noalloc(p, 1, 257, 151936, p, p, p, p, None, p, p, None, 16, None) == ERR_ARG
    assert lib.ddtree_accept_noalloc(p, 64, 1025, 151936, p, p, p, p, p, p, p, None, 16, None) == ERR_WS
    # compact: bad element size
    dst = (ctypes.c_int32 * 1)(0)
    assert lib.ddtree_compact(p, p, p, p, ctypes.cast(dst, ctypes.c_void_p), 1, 17, 8, 1, 64, 3, p, p,
                              None) == ERR_ARG
    assert lib.ddtree_compact(odd, p, p, p, ctypes.cast(dst, ctypes.c_void_p), 1, 17, 8, 1, 64, 2, p, p,
                              None) == ERR_ARG
    # profile hook: bad arguments
    assert lib.ddtree_profile_enable(1 << 20, 4) == ERR_ARG
    assert lib.ddtree_profile_enable_every(1, 4, 0) == ERR_ARG
    assert lib.ddtree_profile_read(99, p, 1) == ERR_ARG
    # the construction selector takes its three values only, and is host-side state
    assert lib.ddtree_set_build_algorithm(3) == ERR_ARG
    assert lib.ddtree_set_build_algorithm(-1) == ERR_ARG
    for algo in (2, 1, 0):
        assert lib.ddtree_set_build_algorithm(algo) == 0
    assert lib.ddtree_build_giveups(None) == ERR_ARG


def test_product_path_does_not_import_the_oracle():
    import ast
    pkg = os.path.join(ROOT, "paper_2604_12989_amd")
    for fn in os.listdir(pkg):
        if fn.endswith(".py"):
            tree = ast.parse(open(os.path.join(pkg, fn)).read())
            for node in ast.walk(tree):
                names = []
                if isinstance(node, ast.Import):
                    names = [a.name for a in node.names]
                elif isinstance(node, ast.ImportFrom):
                    names = [node.module or ""]
                assert not any(n.split(".")[0] == "oracle" for n in names), fn
    for fn in os.listdir(os.path.join(pkg, "csrc")):
        assert "oracle" not in open(os.path.join(pkg, "csrc", fn)).read(), fn
